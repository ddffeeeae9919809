// Device helpers shared by the hash-grid encode kernels: level geometry, cell lookup, corner entries
// and trilinear weights (Sec. 3.2, Sec. 4.1; hash of Instant-NGP Eq. 4).  Internal, not part of the ABI.
#pragma once
#include "dg_internal.h"

namespace dg_encode {

constexpr uint32_t kPrimeY = 2654435761u, kPrimeZ = 805459861u;   // Instant-NGP Eq. 4 (x prime is 1)

struct LevelGeom {
    uint32_t res[3];
    uint32_t dense;
    uint32_t offset;
    float scale[3];
};

__device__ __forceinline__ LevelGeom level_of(const dg_grid_desc &g, uint32_t l)
{
    LevelGeom v;
    v.res[0] = g.res[l][0]; v.res[1] = g.res[l][1]; v.res[2] = g.res[l][2];
    v.dense = g.dense[l];
    v.offset = g.offset[l];
    v.scale[0] = g.scale[l][0]; v.scale[1] = g.scale[l][1]; v.scale[2] = g.scale[l][2];
    return v;
}

// cell and fractional position of a sample at one level; one fp32 multiply, no contraction
__device__ __forceinline__ void locate(const LevelGeom &lv, const float u[3], uint32_t cell[3], float frac[3])
{
#pragma clang fp contract(off)
#pragma unroll
    for (int a = 0; a < 3; ++a) {
        float c = u[a];
        c = c >= 0.0f ? c : 0.0f;     // NaN lands on 0 as well
        c = c > 1.0f ? 1.0f : c;
        const float pos = c * lv.scale[a];
        uint32_t i = (uint32_t)floorf(pos);
        const uint32_t last = lv.res[a] - 1u;
        i = i > last ? last : i;
        cell[a] = i;
        frac[a] = pos - (float)i;
    }
}

// entry indices (relative to the level) of the 8 corners, corner c = cx + 2cy + 4cz
__device__ __forceinline__ void corner_entries(const LevelGeom &lv, uint32_t mask, const uint32_t cell[3], uint32_t e[8])
{
    if (lv.dense) {
        const uint32_t nx = lv.res[0] + 1u, nxy = nx * (lv.res[1] + 1u);
        const uint32_t base = cell[0] + nx * cell[1] + nxy * cell[2];
#pragma unroll
        for (int c = 0; c < 8; ++c) e[c] = base + (c & 1) + ((c >> 1) & 1) * nx + ((c >> 2) & 1) * nxy;
    } else {
        const uint32_t hy0 = cell[1] * kPrimeY, hy1 = hy0 + kPrimeY;
        const uint32_t hz0 = cell[2] * kPrimeZ, hz1 = hz0 + kPrimeZ;
#pragma unroll
        for (int c = 0; c < 8; ++c)
            e[c] = ((cell[0] + (c & 1)) ^ ((c & 2) ? hy1 : hy0) ^ ((c & 4) ? hz1 : hz0)) & mask;
    }
}

__device__ __forceinline__ void corner_weights(const float frac[3], float w[8])
{
    const float wx[2] = {1.0f - frac[0], frac[0]}, wy[2] = {1.0f - frac[1], frac[1]}, wz[2] = {1.0f - frac[2], frac[2]};
#pragma unroll
    for (int c = 0; c < 8; ++c) w[c] = wx[c & 1] * wy[(c >> 1) & 1] * wz[(c >> 2) & 1];
}


// length of the longest run of lanes that share a cell, from the mask of run heads (wavefront-uniform)
__device__ __forceinline__ int longest_run(unsigned long long heads)
{
    unsigned long long inner = ~heads;      // lanes that continue a run
    int len = 1;
    while (inner) { inner &= inner << 1; ++len; }
    return len;
}

}  // namespace dg_encode
