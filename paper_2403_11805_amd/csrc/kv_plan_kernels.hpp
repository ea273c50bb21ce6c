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

}  // namespace kvs
