// The order in which the sampling kernels (masked argmax, masked top-k) rank logits.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace wg {

// float bits -> unsigned integer that orders like the number: NaN lowest (0), then -inf ... +inf;
// -0.0 is folded into +0.0 so that the two compare equal.
__device__ __forceinline__ uint32_t order_key(uint32_t u)
{
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0u;               // NaN
    if ((u << 1) == 0u) u = 0u;                                    // -0.0 == +0.0
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float elem_float(uint32_t raw) { return __uint_as_float(raw); }
__device__ __forceinline__ float elem_float(uint16_t raw) { return __uint_as_float((uint32_t)raw << 16); }  // bfloat16

}  // namespace wg
