// Multi-resolution hash-grid encode: forward gather and backward scatter-add (Sec. 3.2, Sec. 4.1).
//
// Features and their gradients are level-major planes, [L][N][2]: every kernel here walks one level
// at a time and then reads or writes consecutive samples contiguously.
#include "encode_common.h"

namespace {

using namespace dg_encode;

constexpr int kBlock = 256;
// Forward gather, level-major: workgroups are ordered level after level, so at any moment the chip
// works on one level (two at a boundary) and that level's table slice -- at most T entries, 4 MB for
// T = 2^19 -- stays resident in every XCD's L2 while all samples stream past it.  Features are written
// as one plane per level, feat[l][n][2], so the stores of a wavefront are contiguous.
template <bool kHalf>
__global__ void __launch_bounds__(kBlock)
encode_fwd_kernel(dg_grid_desc g, const float2 *__restrict__ table, const float *__restrict__ u, uint64_t N,
                  void *__restrict__ feat, uint32_t n_tiles)
{
    const uint32_t l = blockIdx.x / n_tiles;
    const uint64_t n = (uint64_t)(blockIdx.x % n_tiles) * kBlock + threadIdx.x;
    if (n >= N) return;
    const float uu[3] = {u[3 * n], u[3 * n + 1], u[3 * n + 2]};
    const uint32_t mask = (1u << g.log2_T) - 1u;
    const LevelGeom lv = level_of(g, l);
    uint32_t cell[3], e[8];
    float frac[3], w[8];
    locate(lv, uu, cell, frac);
    corner_entries(lv, mask, cell, e);
    corner_weights(frac, w);
    float2 v[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) v[c] = table[(size_t)lv.offset + e[c]];
    float f0 = 0.0f, f1 = 0.0f;
#pragma unroll
    for (int c = 0; c < 8; ++c) { f0 = fmaf(w[c], v[c].x, f0); f1 = fmaf(w[c], v[c].y, f1); }
    if (kHalf) {
        reinterpret_cast<__half2 *>(feat)[(size_t)l * N + n] = __floats2half2_rn(f0, f1);
    } else {
        reinterpret_cast<float2 *>(feat)[(size_t)l * N + n] = make_float2(f0, f1);
    }
}

// The same with two lanes per sample: lane 2i takes the four corners with cx = 0, lane 2i + 1 those with cx = 1, and a
// DPP move adds the two halves.  The two entries of an x-pair almost always share a cache line, and neighbouring lanes
// that ask for the same line cost the vector cache one look-up instead of two.
template <bool kHalf>
__global__ void __launch_bounds__(kBlock)
encode_fwd_pair_kernel(dg_grid_desc g, const float2 *__restrict__ table, const float *__restrict__ u, uint64_t N,
                       void *__restrict__ feat, uint32_t n_tiles)
{
    const uint32_t l = blockIdx.x / n_tiles;
    const uint64_t s = (uint64_t)(blockIdx.x % n_tiles) * (kBlock / 2) + threadIdx.x / 2;
    const uint32_t cx = threadIdx.x & 1u;
    const bool live = s < N;
    const uint64_t n = live ? s : N - 1;                 // every lane stays in for the exchange
    const float uu[3] = {u[3 * n], u[3 * n + 1], u[3 * n + 2]};
    const uint32_t mask = (1u << g.log2_T) - 1u;
    const LevelGeom lv = level_of(g, l);
    uint32_t cell[3], e[4];
    float frac[3];
    locate(lv, uu, cell, frac);
    if (lv.dense) {
        const uint32_t nx = lv.res[0] + 1u, nxy = nx * (lv.res[1] + 1u);
        const uint32_t base = cell[0] + cx + nx * cell[1] + nxy * cell[2];
#pragma unroll
        for (int k = 0; k < 4; ++k) e[k] = base + (k & 1) * nx + (k >> 1) * nxy;
    } else {
        const uint32_t hy0 = cell[1] * kPrimeY, hy1 = hy0 + kPrimeY;
        const uint32_t hz0 = cell[2] * kPrimeZ, hz1 = hz0 + kPrimeZ;
#pragma unroll
        for (int k = 0; k < 4; ++k) e[k] = ((cell[0] + cx) ^ ((k & 1) ? hy1 : hy0) ^ ((k & 2) ? hz1 : hz0)) & mask;
    }
    const float wx = cx ? frac[0] : 1.0f - frac[0];
    const float wy[2] = {1.0f - frac[1], frac[1]}, wz[2] = {1.0f - frac[2], frac[2]};
    float2 v[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) v[k] = table[(size_t)lv.offset + e[k]];
    float f0 = 0.0f, f1 = 0.0f;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const float w = wx * wy[k & 1] * wz[k >> 1];
        f0 = fmaf(w, v[k].x, f0);
        f1 = fmaf(w, v[k].y, f1);
    }
    // the partner's half: lanes swapped within pairs (quad_perm 1, 0, 3, 2)
    f0 += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(f0), 0xB1, 0xF, 0xF, true));
    f1 += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(f1), 0xB1, 0xF, 0xF, true));
    if (!live || cx) return;
    if (kHalf) {
        reinterpret_cast<__half2 *>(feat)[(size_t)l * N + n] = __floats2half2_rn(f0, f1);
    } else {
        reinterpret_cast<float2 *>(feat)[(size_t)l * N + n] = make_float2(f0, f1);
    }
}

// Backward scatter.  A wavefront holds 64 consecutive samples, i.e. a stretch of one ray, so at the
// coarser levels neighbouring lanes sit in the same cell and add into the same 8 entries.  Global
// fp32 atomics retire at a fixed rate per distinct cache line touched by an instruction, whatever the
// scope or table size, so the kernel spends ALU to shrink that count:
//  * lanes are grouped into runs of equal cell; a segmented wavefront scan sums each run's 16
//    corner x feature values and only the run's last lane issues atomics;
//  * where runs are short (fine levels) the scan is skipped and lane pairs (2k, 2k+1) serve first the
//    even lane's sample, then the odd lane's: the two lanes add the .x and .y of the same entry in one
//    instruction, which the memory pipeline treats as one request.
__global__ void __launch_bounds__(kBlock)
encode_bwd_kernel(dg_grid_desc g, const float *__restrict__ u, const float2 *__restrict__ dfeat, uint64_t N,
                  float *__restrict__ dtable, uint32_t n_groups)
{
    const uint32_t group = blockIdx.x % n_groups;
    const uint64_t n = (uint64_t)(blockIdx.x / n_groups) * kBlock + threadIdx.x;
    const bool live = n < N;
    const uint64_t nn = live ? n : N - 1;
    const int lane = threadIdx.x % dg::kWave;
    const float uu[3] = {u[3 * nn], u[3 * nn + 1], u[3 * nn + 2]};
    const uint32_t mask = (1u << g.log2_T) - 1u;
    for (uint32_t l = group; l < g.n_levels; l += n_groups) {
        const LevelGeom lv = level_of(g, l);
        uint32_t cell[3], e[8];
        float frac[3], w[8];
        locate(lv, uu, cell, frac);
        corner_entries(lv, mask, cell, e);
        corner_weights(frac, w);
        float2 gfe = dfeat[(size_t)l * N + nn];
        if (!live) gfe = make_float2(0.0f, 0.0f);
        float *level_base = dtable + 2 * (size_t)lv.offset;

        // runs of lanes that share a cell
        bool head = lane == 0;
#pragma unroll
        for (int a = 0; a < 3; ++a) head |= from_lane_below(cell[a]) != cell[a];
        const unsigned long long heads = __ballot(head);
        float vx[8], vy[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) { vx[c] = w[c] * gfe.x; vy[c] = w[c] * gfe.y; }

        if (__popcll(heads) <= 40) {
            segmented_sum(vx, vy, head, heads);
            const bool tail = lane == dg::kWave - 1 || ((heads >> ((lane + 1) & 63)) & 1ull);
            if (tail) {
#pragma unroll
                for (int c = 0; c < 8; ++c) {
                    if (vx[c] != 0.0f) unsafeAtomicAdd(level_base + 2 * (size_t)e[c], vx[c]);
                    if (vy[c] != 0.0f) unsafeAtomicAdd(level_base + 2 * (size_t)e[c] + 1, vy[c]);
                }
            }
        } else {
            const int sub = lane & 1;
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                // even lane's sample: even lane adds x, odd lane adds the even lane's y
                const uint32_t e_dn = __shfl_up(e[c], 1, dg::kWave);
                const float y_dn = __shfl_up(vy[c], 1, dg::kWave);
                const uint32_t ea = sub ? e_dn : e[c];
                const float va = sub ? y_dn : vx[c];
                if (va != 0.0f) unsafeAtomicAdd(level_base + 2 * (size_t)ea + sub, va);
                // odd lane's sample: even lane adds the odd lane's x, odd lane adds its own y
                const uint32_t e_up = __shfl_down(e[c], 1, dg::kWave);
                const float x_up = __shfl_down(vx[c], 1, dg::kWave);
                const uint32_t eb = sub ? e[c] : e_up;
                const float vb = sub ? vy[c] : x_up;
                if (vb != 0.0f) unsafeAtomicAdd(level_base + 2 * (size_t)eb + sub, vb);
            }
        }
    }
}

__global__ void __launch_bounds__(kBlock)
corner_index_kernel(dg_grid_desc g, const float *__restrict__ u, uint64_t N, uint32_t *__restrict__ idx)
{
    const uint64_t t = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (t >= N * g.n_levels) return;
    const uint64_t n = t / g.n_levels;
    const uint32_t l = (uint32_t)(t % g.n_levels);
    const float uu[3] = {u[3 * n], u[3 * n + 1], u[3 * n + 2]};
    const LevelGeom lv = level_of(g, l);
    uint32_t cell[3], e[8];
    float frac[3];
    locate(lv, uu, cell, frac);
    corner_entries(lv, (1u << g.log2_T) - 1u, cell, e);
#pragma unroll
    for (int c = 0; c < 8; ++c) idx[t * 8 + c] = lv.offset + e[c];
}

int check_desc(const dg_grid_desc *d, const char *who)
{
    DG_REQUIRE(d, DG_ERR_ARG, "%s: null descriptor", who);
    DG_REQUIRE(d->n_levels >= 1 && d->n_levels <= DG_MAX_LEVELS && d->n_features == 2 && d->log2_T <= 24,
               DG_ERR_UNSUPPORTED, "%s: unsupported grid (L=%u F=%u log2_T=%u)", who, d->n_levels, d->n_features, d->log2_T);
    for (uint32_t l = 0; l < d->n_levels; ++l) {
        const uint64_t verts = (uint64_t)(d->res[l][0] + 1) * (d->res[l][1] + 1) * (d->res[l][2] + 1);
        const uint64_t len = (uint64_t)d->offset[l + 1] - d->offset[l];
        DG_REQUIRE(d->res[l][0] >= 1 && d->res[l][1] >= 1 && d->res[l][2] >= 1, DG_ERR_ARG, "%s: empty level %u", who, l);
        DG_REQUIRE(d->offset[l + 1] > d->offset[l] && (d->dense[l] ? verts <= len : len == (1ull << d->log2_T)),
                   DG_ERR_ARG, "%s: level %u does not fit its table slice", who, l);
    }
    DG_REQUIRE(d->offset[d->n_levels] == d->n_entries, DG_ERR_ARG, "%s: n_entries disagrees with offsets", who);
    return DG_OK;
}

int grid_for(uint64_t N, uint32_t n_groups, uint32_t *n_blocks, const char *who)
{
    const uint64_t tiles = (N + kBlock - 1) / kBlock;
    DG_REQUIRE(tiles * n_groups <= 0x7fffffffull, DG_ERR_UNSUPPORTED, "%s: N too large for one launch", who);
    *n_blocks = (uint32_t)(tiles * n_groups);
    return DG_OK;
}

}  // namespace

extern "C" int dg_hashgrid_encode_fwd(const dg_grid_desc *desc, const float *table, const float *u, uint64_t N,
                                      void *feat, uint32_t feat_dtype, void *stream)
{
    if (int rc = check_desc(desc, "dg_hashgrid_encode_fwd")) return rc;
    DG_REQUIRE(feat_dtype == DG_F32 || feat_dtype == DG_F16, DG_ERR_ARG, "dg_hashgrid_encode_fwd: bad feat_dtype");
    if (N == 0) return DG_OK;
    DG_REQUIRE(table && u && feat, DG_ERR_ARG, "dg_hashgrid_encode_fwd: null pointer");
    DG_REQUIRE(dg::aligned(table, 8) && dg::aligned(feat, feat_dtype == DG_F16 ? 4 : 8), DG_ERR_ARG,
               "dg_hashgrid_encode_fwd: table/feat misaligned");
    uint32_t n_blocks;
    hipStream_t st = (hipStream_t)stream;
    // Two lanes per sample while the tables are small enough to be served from cache (c2, T = 2^19: 3.09 -> 2.33 ms;
    // T = 2^22: 9 % faster); with T = 2^24 the gather waits for HBM and the spare lanes only cost (3 % slower).
    if (desc->log2_T <= 22) {
        if (int rc = grid_for(2 * N, desc->n_levels, &n_blocks, "dg_hashgrid_encode_fwd")) return rc;
        const uint32_t n_tiles = n_blocks / desc->n_levels;
        if (feat_dtype == DG_F16)
            encode_fwd_pair_kernel<true><<<n_blocks, kBlock, 0, st>>>(*desc, (const float2 *)table, u, N, feat, n_tiles);
        else
            encode_fwd_pair_kernel<false><<<n_blocks, kBlock, 0, st>>>(*desc, (const float2 *)table, u, N, feat, n_tiles);
        return dg::launch_status("dg_hashgrid_encode_fwd");
    }
    if (int rc = grid_for(N, desc->n_levels, &n_blocks, "dg_hashgrid_encode_fwd")) return rc;
    const uint32_t n_tiles = n_blocks / desc->n_levels;
    if (feat_dtype == DG_F16)
        encode_fwd_kernel<true><<<n_blocks, kBlock, 0, st>>>(*desc, (const float2 *)table, u, N, feat, n_tiles);
    else
        encode_fwd_kernel<false><<<n_blocks, kBlock, 0, st>>>(*desc, (const float2 *)table, u, N, feat, n_tiles);
    return dg::launch_status("dg_hashgrid_encode_fwd");
}

extern "C" size_t dg_hashgrid_encode_bwd_workspace_bytes(const dg_grid_desc *desc, uint64_t N)
{
    if (check_desc(desc, "dg_hashgrid_encode_bwd_workspace_bytes")) return 0;
    return dg::encode_bwd_binned_workspace_bytes(desc, N);
}

extern "C" int dg_hashgrid_encode_bwd_count(const dg_grid_desc *desc, const float *u, uint64_t N, void *ws, size_t ws_bytes,
                                            void *stream)
{
    if (int rc = check_desc(desc, "dg_hashgrid_encode_bwd_count")) return rc;
    if (N == 0) return DG_OK;
    DG_REQUIRE(u && ws, DG_ERR_ARG, "dg_hashgrid_encode_bwd_count: null pointer");
    DG_REQUIRE(dg::aligned(ws, 256), DG_ERR_ARG, "dg_hashgrid_encode_bwd_count: workspace must be 256-byte aligned");
    return dg::encode_bwd_binned_count(desc, u, N, ws, ws_bytes, (hipStream_t)stream);
}

namespace {
int encode_bwd(const dg_grid_desc *desc, const float *u, const float *dfeat, uint64_t N, float *dtable, void *ws, size_t ws_bytes,
               bool counted, void *stream)
{
    if (int rc = check_desc(desc, "dg_hashgrid_encode_bwd")) return rc;
    if (N == 0) return DG_OK;
    DG_REQUIRE(u && dfeat && dtable, DG_ERR_ARG, "dg_hashgrid_encode_bwd: null pointer");
    DG_REQUIRE(dg::aligned(dfeat, 8) && dg::aligned(dtable, 8), DG_ERR_ARG, "dg_hashgrid_encode_bwd: misaligned pointer");
    DG_REQUIRE(ws || !counted, DG_ERR_ARG, "dg_hashgrid_encode_bwd_counted: the workspace that holds the counts is missing");
    if (ws) {
        DG_REQUIRE(dg::aligned(ws, 256), DG_ERR_ARG, "dg_hashgrid_encode_bwd: workspace must be 256-byte aligned");
        return dg::encode_bwd_binned(desc, u, dfeat, N, dtable, ws, ws_bytes, counted, (hipStream_t)stream);
    }
    const uint32_t n_groups = desc->n_levels < 8 ? desc->n_levels : 8;
    uint32_t n_blocks;
    if (int rc = grid_for(N, n_groups, &n_blocks, "dg_hashgrid_encode_bwd")) return rc;
    encode_bwd_kernel<<<n_blocks, kBlock, 0, (hipStream_t)stream>>>(*desc, u, (const float2 *)dfeat, N, dtable, n_groups);
    return dg::launch_status("dg_hashgrid_encode_bwd");
}
}  // namespace

extern "C" int dg_hashgrid_encode_bwd(const dg_grid_desc *desc, const float *u, const float *dfeat, uint64_t N,
                                      float *dtable, void *ws, size_t ws_bytes, void *stream)
{
    return encode_bwd(desc, u, dfeat, N, dtable, ws, ws_bytes, false, stream);
}

extern "C" int dg_hashgrid_encode_bwd_counted(const dg_grid_desc *desc, const float *u, const float *dfeat, uint64_t N,
                                              float *dtable, void *ws, size_t ws_bytes, void *stream)
{
    return encode_bwd(desc, u, dfeat, N, dtable, ws, ws_bytes, true, stream);
}

extern "C" int dg_hashgrid_corner_indices(const dg_grid_desc *desc, const float *u, uint64_t N, uint32_t *idx,
                                          void *stream)
{
    if (int rc = check_desc(desc, "dg_hashgrid_corner_indices")) return rc;
    if (N == 0) return DG_OK;
    DG_REQUIRE(u && idx, DG_ERR_ARG, "dg_hashgrid_corner_indices: null pointer");
    const uint64_t n_blocks = (N * desc->n_levels + kBlock - 1) / kBlock;
    DG_REQUIRE(n_blocks <= 0x7fffffffull, DG_ERR_UNSUPPORTED, "dg_hashgrid_corner_indices: N too large");
    corner_index_kernel<<<(uint32_t)n_blocks, kBlock, 0, (hipStream_t)stream>>>(*desc, u, N, idx);
    return dg::launch_status("dg_hashgrid_corner_indices");
}
