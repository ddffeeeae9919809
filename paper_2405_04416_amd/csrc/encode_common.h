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


// value of the lane below (lane - 1) in the wavefront; lane 0 gets its own.  A DPP move: no LDS traffic, no wait.
__device__ __forceinline__ uint32_t from_lane_below(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x138 /* wave_shr:1 */, 0xF, 0xF, false);
}

// length of the longest run of lanes that share a cell, from the mask of run heads (wavefront-uniform)
__device__ __forceinline__ int longest_run(unsigned long long heads)
{
    unsigned long long inner = ~heads;      // lanes that continue a run
    int len = 1;
    while (inner) { inner &= inner << 1; ++len; }
    return len;
}

// ---- segmented sum over the wavefront with DPP moves (no LDS traffic, no waits) ----------------------
// Lanes form runs (a run starts where `head` is set; lane 0 always starts one).  After the call the last
// lane of every run holds the sum of that run's 16 values.  One step combines each lane with a lane
// further down: (v, f) <- (f ? v : v + v_src, f | f_src), f meaning "a run start lies in the span summed so
// far".  Steps: row_shr 1, 2, 4, 8 inside rows of 16 lanes, then row_bcast:15 into rows 1 and 3 and
// row_bcast:31 into rows 2 and 3 -- the classic wavefront scan, made segment-aware.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ void seg_step(float (&vx)[8], float (&vy)[8], int &f)
{
    const int fs = __builtin_amdgcn_update_dpp(0, f, CTRL, ROW_MASK, 0xF, true);
    const float take = f ? 0.0f : 1.0f;      // v + 1 * t is exact, so one multiply-add (which can carry the DPP move) does the step
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        const float tx = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(vx[c]), CTRL, ROW_MASK, 0xF, true));
        const float ty = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(vy[c]), CTRL, ROW_MASK, 0xF, true));
        vx[c] = __builtin_fmaf(tx, take, vx[c]);
        vy[c] = __builtin_fmaf(ty, take, vy[c]);
    }
    f |= fs;
}

__device__ __forceinline__ void segmented_sum(float (&vx)[8], float (&vy)[8], bool head, unsigned long long heads)
{
    int f = head ? 1 : 0;
    const int longest = longest_run(heads);         // wavefront-uniform: steps a run of that length cannot need are skipped
    if (longest > 1) seg_step<0x111, 0xF>(vx, vy, f);
    if (longest > 2) seg_step<0x112, 0xF>(vx, vy, f);
    if (longest > 4) seg_step<0x114, 0xF>(vx, vy, f);
    if (longest > 8) seg_step<0x118, 0xF>(vx, vy, f);
    if (!((heads >> 16) & 1ull) || !((heads >> 48) & 1ull)) seg_step<0x142, 0xA>(vx, vy, f);
    if (!((heads >> 32) & 1ull)) seg_step<0x143, 0xC>(vx, vy, f);
}

}  // namespace dg_encode
