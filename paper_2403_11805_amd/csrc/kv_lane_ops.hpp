// Cross-lane helpers shared by the kernels of libkvswitch (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kvs {

// Exchange between lanes l and l ^ 32 of a wavefront.
// v_permlane32_swap returns (low half in both halves, high half in both halves),
// so one VALU-speed instruction plus the combining op gives every lane the
// reduction over both halves, with no trip through the LDS crossbar.
typedef unsigned int xh_u2_t __attribute__((ext_vector_type(2)));
// (The vector elements are copied to scalars before the bit casts: a bit cast
// applied directly to a vector element reads element 0.)
__device__ __forceinline__ void xhalf_both_u32(unsigned int u, unsigned int& lo, unsigned int& hi) {
    const xh_u2_t r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    lo = r.x;
    hi = r.y;
}
__device__ __forceinline__ void xhalf_both(float v, float& lo, float& hi) {
    const unsigned int u = __builtin_bit_cast(unsigned int, v);
    const xh_u2_t r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    const unsigned int rx = r.x, ry = r.y;
    lo = __builtin_bit_cast(float, rx);
    hi = __builtin_bit_cast(float, ry);
}
__device__ __forceinline__ float xhalf_max(float v) {
    float lo, hi;
    xhalf_both(v, lo, hi);
    return fmaxf(lo, hi);
}
__device__ __forceinline__ float xhalf_min(float v) {
    float lo, hi;
    xhalf_both(v, lo, hi);
    return fminf(lo, hi);
}
__device__ __forceinline__ float xhalf_sum(float v) {
    float lo, hi;
    xhalf_both(v, lo, hi);
    return lo + hi;
}

}  // namespace kvs
