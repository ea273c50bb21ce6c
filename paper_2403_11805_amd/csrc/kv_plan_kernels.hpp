// Widths, record offsets and the whole-cache gather list computed on the device
// (Sec. 3.2, Eq. 2 with fixed thresholds; Sec. 3.1, Load primitive): the same
// integers as the host functions produce, for callers that keep scoring,
// compression and swap-in on one stream without a host round trip.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kvs {

constexpr int kPlanRankThreads = 256;
constexpr int kPlanScanThreads = 1024;

// Record bytes by bit-width (0 where the width is not one of the format's).
struct RecordBytes {
    uint64_t w16, w8, w4, w2, w1;
    __device__ __forceinline__ uint64_t of(int b) const {
        return b == 8 ? w8 : (b == 4 ? w4 : (b == 2 ? w2 : (b == 16 ? w16 : (b == 1 ? w1 : 0))));
    }
};

// Chunk i's rank in the order (density descending, index ascending) by counting
// the chunks that come before it; the rank decides the width.  One thread per
// chunk, densities of the others passed through LDS a tile at a time (every
// lane reads the same word: a broadcast).
__global__ __launch_bounds__(kPlanRankThreads) void plan_bits_kernel(
    const float* __restrict__ density, int n, int k8, int k84, int chunk_tokens,
    uint8_t* __restrict__ bits, int32_t* __restrict__ dst_tok) {
    __shared__ float tile[kPlanRankThreads];
    const int i = blockIdx.x * kPlanRankThreads + threadIdx.x;
    const float di = density[i < n ? i : n - 1];
    int rank = 0;
    for (int base = 0; base < n; base += kPlanRankThreads) {
        const int j0 = base + threadIdx.x;
        __syncthreads();
        tile[threadIdx.x] = density[j0 < n ? j0 : n - 1];
        __syncthreads();
        const int lim = n - base < kPlanRankThreads ? n - base : kPlanRankThreads;
        for (int jj = 0; jj < lim; ++jj) {
            const float dj = tile[jj];
            // j comes before i: denser, or neither denser than the other and earlier
            const bool before = dj > di || (!(di > dj) && base + jj < i);
            rank += before ? 1 : 0;
        }
    }
    if (i < n) {
        bits[i] = static_cast<uint8_t>(rank < k8 ? 8 : (rank < k84 ? 4 : 2));
        dst_tok[i] = i * chunk_tokens;
    }
}

// off[0] = 0, off[i + 1] = off[i] + record bytes of chunk i.  One workgroup; each
// thread owns a run of consecutive chunks, the run totals are scanned through LDS.
__global__ __launch_bounds__(kPlanScanThreads) void plan_offsets_kernel(
    const uint8_t* __restrict__ bits, int n, RecordBytes rec, uint64_t* __restrict__ off) {
    __shared__ uint64_t part[kPlanScanThreads];
    const int tid = threadIdx.x;
    const int per = (n + kPlanScanThreads - 1) / kPlanScanThreads;
    const int begin = tid * per < n ? tid * per : n;
    const int end = begin + per < n ? begin + per : n;
    uint64_t sum = 0;
    for (int i = begin; i < end; ++i) sum += rec.of(bits[i]);
    part[tid] = sum;
    __syncthreads();
    for (int d = 1; d < kPlanScanThreads; d <<= 1) {      // inclusive scan of the run totals
        const uint64_t add = tid >= d ? part[tid - d] : 0;
        __syncthreads();
        part[tid] += add;
        __syncthreads();
    }
    uint64_t at = part[tid] - sum;                          // bytes before this thread's run
    for (int i = begin; i < end; ++i) {
        off[i] = at;
        at += rec.of(bits[i]);
    }
    if (tid == kPlanScanThreads - 1) off[n] = part[tid];
}

// Both steps in one workgroup for up to kPlanScanThreads chunks: a single launch between
// scoring and compression.  `width` = n rounded up to whole wavefronts; the block has
// parts * width threads (parts a power of two, at most 16): thread (part, i) counts the chunks
// that come before chunk i among its share of the others, part 0 adds the counts up and goes on
// alone (one chunk per thread).
__global__ __launch_bounds__(kPlanScanThreads) void plan_small_kernel(
    const float* __restrict__ density, int n, int width, int k8, int k84, int chunk_tokens, RecordBytes rec,
    uint8_t* __restrict__ bits, uint64_t* __restrict__ off, int32_t* __restrict__ dst_tok) {
    __shared__ __attribute__((aligned(16))) float dens[kPlanScanThreads];
    __shared__ uint64_t part[kPlanScanThreads];
    __shared__ int counts[kPlanScanThreads];
    const int parts = static_cast<int>(blockDim.x) / width;
    const int i = static_cast<int>(threadIdx.x) % width, q = static_cast<int>(threadIdx.x) / width;
    const float di = density[i < n ? i : n - 1];
    if (q == 0) dens[i] = i < n ? di : -__builtin_inff();          // padding never comes before a chunk
    __syncthreads();
    const int span = width / parts;                                 // a multiple of 4: width of 64, parts <= 16
    int rank = 0;
    for (int j = q * span; j < (q + 1) * span; j += 4) {
        const float4 d4 = *reinterpret_cast<const float4*>(dens + j);
        rank += (d4.x > di || (!(di > d4.x) && j + 0 < i)) ? 1 : 0;
        rank += (d4.y > di || (!(di > d4.y) && j + 1 < i)) ? 1 : 0;
        rank += (d4.z > di || (!(di > d4.z) && j + 2 < i)) ? 1 : 0;
        rank += (d4.w > di || (!(di > d4.w) && j + 3 < i)) ? 1 : 0;
    }
    counts[threadIdx.x] = rank;
    __syncthreads();
    rank = 0;
    for (int p = 0; p < parts; ++p) rank += counts[p * width + i];
    const int b = rank < k8 ? 8 : (rank < k84 ? 4 : 2);
    const uint64_t own = (q == 0 && i < n) ? rec.of(b) : 0;
    if (q == 0) part[i] = own;
    __syncthreads();
    for (int d = 1; d < width; d <<= 1) {
        const uint64_t add = (q == 0 && i >= d) ? part[i - d] : 0;
        __syncthreads();
        if (q == 0) part[i] += add;
        __syncthreads();
    }
    if (q == 0 && i < n) {
        bits[i] = static_cast<uint8_t>(b);
        dst_tok[i] = i * chunk_tokens;
        off[i] = part[i] - own;
        if (i == n - 1) off[n] = part[i];
    }
}

// ------------------------------------------------------------------ thresholds from a global ratio (Eq. 2-3)

constexpr int kPlanOptMaxChunks = 8192;      // sorted densities of one context held in LDS as doubles

// Rank of every chunk as in plan_bits_kernel, written out with the densities in rank order:
// rank_out[i] = rank of chunk i, sorted_out[rank] = density of chunk i as a double.  Ranks are a
// permutation, so every slot of sorted_out is written exactly once.
__global__ __launch_bounds__(kPlanRankThreads) void plan_rank_kernel(
    const float* __restrict__ density, int n, int32_t* __restrict__ rank_out, double* __restrict__ sorted_out) {
    __shared__ float tile[kPlanRankThreads];
    const int i = blockIdx.x * kPlanRankThreads + threadIdx.x;
    const float di = density[i < n ? i : n - 1];
    int rank = 0;
    for (int base = 0; base < n; base += kPlanRankThreads) {
        const int j0 = base + threadIdx.x;
        __syncthreads();
        tile[threadIdx.x] = density[j0 < n ? j0 : n - 1];
        __syncthreads();
        const int lim = n - base < kPlanRankThreads ? n - base : kPlanRankThreads;
        for (int jj = 0; jj < lim; ++jj) {
            const float dj = tile[jj];
            const bool before = dj > di || (!(di > dj) && base + jj < i);
            rank += before ? 1 : 0;
        }
    }
    if (i < n) {
        rank_out[i] = rank;
        sorted_out[rank] = static_cast<double>(di);
    }
}

// Eq. 3 over the ranked densities, then widths, offsets and the gather list; one workgroup of
// kPlanScanThreads threads, n <= kPlanOptMaxChunks.
//   sorted_off : in: the n densities in rank order as doubles (plan_rank_kernel); out: the n + 1
//                record offsets (the same buffer: every density is in LDS before an offset is written)
//   rank_dst   : in: rank of chunk i; out: dst_tok[i] = i * chunk_tokens
// The sums are those of the host function, bit for bit: prefix[k] = the k densest added one by one in
// rank order in double (one thread: a chain of n additions), and for every feasible k8 in
// [k8_lo, k8_hi] ctxInfo = w8*S8 + w4*S4 + w2*S2 with S4 = prefix[k8+k4] - prefix[k8], S2 = prefix[n] -
// prefix[k8+k4], k4 = M - 3*k8; the largest value wins, the smallest k8 among equal ones.
__global__ __launch_bounds__(kPlanScanThreads) void plan_optimise_kernel(
    int n, int64_t M, int k8_lo, int k8_hi, double w4, double w2, int chunk_tokens, RecordBytes rec,
    uint64_t* __restrict__ sorted_off, int32_t* __restrict__ rank_dst, uint8_t* __restrict__ bits,
    int32_t* __restrict__ counts) {
    __shared__ double prefix[kPlanOptMaxChunks + 1];
    __shared__ double best_v[kPlanScanThreads / 64];
    __shared__ int best_k[kPlanScanThreads / 64];
    __shared__ uint64_t part[kPlanScanThreads];
    __shared__ int chosen_k8;
    const int tid = threadIdx.x;
    const double* sorted = reinterpret_cast<const double*>(sorted_off);
    for (int k = tid; k < n; k += kPlanScanThreads) prefix[k + 1] = sorted[k];
    __syncthreads();
    if (tid == 0) {
        double acc = 0.0;
        prefix[0] = 0.0;
        for (int k = 1; k <= n; ++k) {
            acc += prefix[k];
            prefix[k] = acc;
        }
    }
    __syncthreads();
    // every feasible k8, strided over the threads; a thread keeps the first of its equal maxima
    double bv = 0.0;
    int bk = -1;
    for (int k8 = k8_lo + tid; k8 <= k8_hi; k8 += kPlanScanThreads) {
        const int k4 = static_cast<int>(M - 3 * static_cast<int64_t>(k8));
        const double s8 = prefix[k8];
        const double s4 = prefix[k8 + k4] - prefix[k8];
        const double s2 = prefix[n] - prefix[k8 + k4];
        const double info = 1.0 * s8 + w4 * s4 + w2 * s2;
        if (bk < 0 || info > bv) {
            bv = info;
            bk = k8;
        }
    }
    // (value, smallest k8) maximum over the wavefront, then over the workgroup
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        const double ov = __shfl_xor(bv, o);
        const int ok = __shfl_xor(bk, o);
        const bool take = ok >= 0 && (bk < 0 || ov > bv || (ov == bv && ok < bk));
        if (take) {
            bv = ov;
            bk = ok;
        }
    }
    if ((tid & 63) == 0) {
        best_v[tid >> 6] = bv;
        best_k[tid >> 6] = bk;
    }
    __syncthreads();
    if (tid == 0) {
        double v = best_v[0];
        int k = best_k[0];
        for (int w = 1; w < kPlanScanThreads / 64; ++w) {
            const double ov = best_v[w];
            const int ok = best_k[w];
            if (ok >= 0 && (k < 0 || ov > v || (ov == v && ok < k))) {
                v = ov;
                k = ok;
            }
        }
        chosen_k8 = k;
        if (counts) {
            const int k4 = static_cast<int>(M - 3 * static_cast<int64_t>(k));
            counts[0] = k;
            counts[1] = k4;
            counts[2] = n - k - k4;
        }
    }
    __syncthreads();
    const int k8 = chosen_k8;
    const int k84 = k8 + static_cast<int>(M - 3 * static_cast<int64_t>(k8));
    // widths from the ranks, offsets by a scan of the record sizes (each thread owns a run of chunks)
    const int per = (n + kPlanScanThreads - 1) / kPlanScanThreads;
    const int begin = tid * per < n ? tid * per : n;
    const int end = begin + per < n ? begin + per : n;
    uint64_t sum = 0;
    for (int i = begin; i < end; ++i) {
        const int r = rank_dst[i];
        const int b = r < k8 ? 8 : (r < k84 ? 4 : 2);
        bits[i] = static_cast<uint8_t>(b);
        rank_dst[i] = i * chunk_tokens;
        sum += rec.of(b);
    }
    part[tid] = sum;
    __syncthreads();
    for (int d = 1; d < kPlanScanThreads; d <<= 1) {
        const uint64_t add = tid >= d ? part[tid - d] : 0;
        __syncthreads();
        part[tid] += add;
        __syncthreads();
    }
    uint64_t at = part[tid] - sum;
    for (int i = begin; i < end; ++i) {
        sorted_off[i] = at;
        const int b = bits[i];                   // this thread's own store above
        at += rec.of(b);
    }
    if (tid == kPlanScanThreads - 1) sorted_off[n] = part[tid];
}

}  // namespace kvs
