// Device helpers shared by the two samplers (fixed stratified and occupancy-guided): the counter-based random
// numbers and the box a sample's unit coordinates refer to.  Internal, not part of the ABI.
#pragma once
#include "dg_internal.h"

namespace dg_sample {

// 64 random bits for (seed, counter): the splitmix64 output mix of seed + golden * (counter + 1)
__device__ __forceinline__ uint64_t mix64(uint64_t seed, uint64_t ctr)
{
    uint64_t z = seed + 0x9E3779B97F4A7C15ull * (ctr + 1ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

__device__ __forceinline__ float unit_float(uint64_t z) { return (float)(uint32_t)(z >> 40) * (1.0f / 16777216.0f); }

// jitter of stratum s of the segment in slot `slot` of ray `ray`
__device__ __forceinline__ float counter_jitter(uint64_t seed, uint32_t ray, uint32_t slot, uint32_t s)
{
    return unit_float(mix64(seed, ((uint64_t)ray << 32) | ((uint64_t)(slot & 0xffffu) << 16) | (uint64_t)(s & 0xffffu)));
}

struct BoxArgs { float lo[3], inv_ext[3]; };

}  // namespace dg_sample
