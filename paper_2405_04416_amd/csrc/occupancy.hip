// Occupancy grid and occupancy-guided sampling (Sec. 3.2: per-voxel densities let marching skip empty space;
// Sec. 4.1: the grid is deformable like the hash grid; Sec. 5.1: its hyper-parameters; refresh rule of
// Instant-NGP App. E.2: decay, candidate cells, maximum, threshold).
//
// Marching: one 64-lane wavefront per segment, one stratum per lane and pass.  The lanes of a pass lie next to
// each other on the ray, so their bit lookups fall into a few cache lines of a bit field that stays in L2
// (512 x 512 x 64 cells are 2 MiB).  Kept samples are compacted with a ballot; segments are placed by an
// exclusive scan over their sample counts, so the layout is deterministic: count, scan, write.
//
// Cells, bits and sample counts are decided in fp32 with one rounding per operation (built with
// -ffp-contract=off).
#include "dg_internal.h"
#include "sample_common.h"
#include <cmath>
#include <cstring>

#pragma clang fp contract(off)

namespace {

using dg_sample::BoxArgs;
using dg_sample::counter_jitter;
using dg_sample::mix64;
using dg_sample::unit_float;

constexpr int kBlock = 256;
constexpr int kWavesPerBlock = kBlock / dg::kWave;
constexpr int kScanItems = 8;                          // values per thread
constexpr int kScanTile = kBlock * kScanItems;         // values per workgroup of the scan
constexpr int kSumsBlock = 1024;

struct OccArgs { uint32_t res[3]; uint32_t n_cells; float scale[3]; };

__device__ __forceinline__ uint32_t cell_of(const OccArgs &g, const float (&u)[3])
{
    uint32_t c[3];
#pragma unroll
    for (int a = 0; a < 3; ++a) {
        float v = u[a];
        v = v >= 0.0f ? v : 0.0f;          // NaN lands on 0 as well
        v = v > 1.0f ? 1.0f : v;
        const float pos = v * g.scale[a];
        uint32_t i = (uint32_t)floorf(pos);
        const uint32_t last = g.res[a] - 1u;
        c[a] = i > last ? last : i;
    }
    return c[0] + g.res[0] * (c[1] + g.res[1] * c[2]);
}

__device__ __forceinline__ bool bit_of(const uint32_t *__restrict__ bits, uint32_t c) { return (bits[c >> 5] >> (c & 31u)) & 1u; }

// ---------------------------------------------------------------- refresh
__device__ __forceinline__ uint64_t candidate_counter(uint32_t iteration, uint32_t i, uint32_t attempt, uint32_t q)
{
    return ((uint64_t)iteration << 36) | ((uint64_t)i << 8) | ((uint64_t)attempt << 2) | q;
}

__global__ void __launch_bounds__(kBlock)
candidates_kernel(OccArgs g, const uint32_t *__restrict__ bits, uint32_t i0, uint32_t M, uint32_t n_uniform, int warmup,
                  uint64_t seed, uint32_t iteration, uint32_t tries, uint32_t *__restrict__ cell, float *__restrict__ u)
{
    const uint32_t j = blockIdx.x * kBlock + threadIdx.x;       // position in this call's output
    if (j >= M) return;
    const uint32_t i = i0 + j;                                   // index of the candidate within the refresh
    uint32_t c = i, attempt = 0;
    if (!warmup) {
        const uint32_t allowed = i < n_uniform ? 1u : tries;
        for (attempt = 0; attempt < allowed; ++attempt) {
            const uint64_t z = mix64(seed, candidate_counter(iteration, i, attempt, 0));
            c = (uint32_t)(((z >> 32) * (uint64_t)g.n_cells) >> 32);
            if (i < n_uniform || bit_of(bits, c)) break;
        }
        if (attempt == allowed) attempt = allowed - 1u;     // no occupied cell met: the last draw stands
    }
    cell[j] = c;
    const uint32_t idx[3] = {c % g.res[0], (c / g.res[0]) % g.res[1], c / (g.res[0] * g.res[1])};
#pragma unroll
    for (uint32_t a = 0; a < 3; ++a) {
        const float xi = unit_float(mix64(seed, candidate_counter(iteration, i, attempt, a + 1u)));
        u[3 * (size_t)j + a] = ((float)idx[a] + xi) / g.scale[a];
    }
}

__global__ void __launch_bounds__(kBlock)
decay_kernel(float *__restrict__ density, uint32_t n_cells, float factor)
{
    const uint32_t c = blockIdx.x * kBlock + threadIdx.x;
    if (c < n_cells) density[c] = density[c] * factor;
}

// densities are >= 0, so their bit patterns order like unsigned integers and the maximum is one integer atomic
__global__ void __launch_bounds__(kBlock)
update_kernel(float *__restrict__ density, uint32_t n_cells, const uint32_t *__restrict__ cell, const float *__restrict__ sigma,
              uint32_t M)
{
    const uint32_t i = blockIdx.x * kBlock + threadIdx.x;
    if (i >= M) return;
    const uint32_t c = cell[i];
    const float s = sigma[i];
    if (c < n_cells && s > 0.0f) atomicMax(reinterpret_cast<unsigned int *>(density) + c, __float_as_uint(s));
}

constexpr int kBitsRounds = 16;                        // cells per thread of the bit-field pass

// one workgroup thresholds kBlock * kBitsRounds consecutive cells; set bits are counted per workgroup, so the shared
// counter takes one atomic per 4096 cells (same-address atomics serialise)
__global__ void __launch_bounds__(kBlock)
bits_kernel(const float *__restrict__ density, uint32_t n_cells, float threshold, uint32_t *__restrict__ bits,
            uint32_t *__restrict__ n_set)
{
    __shared__ uint32_t wave_count[kWavesPerBlock];
    const uint32_t n_words = (n_cells + 31u) >> 5;
    uint32_t mine = 0;
#pragma unroll 4
    for (int round = 0; round < kBitsRounds; ++round) {
        // n_cells <= 2^31 and the grid covers it once: no wrap
        const uint32_t c = (blockIdx.x * kBitsRounds + round) * kBlock + threadIdx.x;
        const bool on = c < n_cells && density[c] > threshold;
        const unsigned long long mask = __ballot(on);
        if (threadIdx.x % dg::kWave == 0 && c < n_cells) {
            const uint32_t w = c >> 5;
            bits[w] = (uint32_t)mask;
            if (w + 1u < n_words) bits[w + 1u] = (uint32_t)(mask >> 32);
            mine += (uint32_t)__popcll(mask);
        }
    }
    if (!n_set) return;
    if (threadIdx.x % dg::kWave == 0) wave_count[threadIdx.x / dg::kWave] = mine;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t total = 0;
        for (int w = 0; w < kWavesPerBlock; ++w) total += wave_count[w];
        if (total) atomicAdd(n_set, total);
    }
}

// ---------------------------------------------------------------- marching
struct MarchOut { float *u, *delta, *t; uint32_t *sample_ray; };

template <bool WRITE>
__global__ void __launch_bounds__(kBlock)
march_kernel(const float *__restrict__ o, const float *__restrict__ d, const float *__restrict__ seg_t,
             const uint32_t *__restrict__ seg_ray, const uint32_t *__restrict__ seg_slot, uint32_t n_seg, uint32_t k_max,
             BoxArgs box, OccArgs occ, const uint32_t *__restrict__ bits, float dt, uint32_t max_steps, uint64_t seed,
             uint32_t capacity, uint32_t *__restrict__ first, MarchOut out, uint32_t *__restrict__ status)
{
    const uint32_t j = blockIdx.x * kWavesPerBlock + threadIdx.x / dg::kWave;
    const uint32_t lane = threadIdx.x % dg::kWave;
    if (!WRITE && blockIdx.x == 0 && threadIdx.x == 0) first[n_seg] = 0;     // the scan turns it into the total
    if (j >= n_seg) return;
    const uint32_t r = seg_ray[j], k = seg_slot[j];
    const float t_in = seg_t[((size_t)r * k_max + k) * 2], t_out = seg_t[((size_t)r * k_max + k) * 2 + 1];
    const float len = t_out - t_in;
    const float wanted = ceilf(len / dt);                   // strata no wider than the marching step
    const uint32_t n = wanted >= (float)max_steps ? max_steps : (wanted >= 1.0f ? (uint32_t)wanted : 1u);
    const float width = len / (float)n;
    const float oo[3] = {o[3 * (size_t)r], o[3 * (size_t)r + 1], o[3 * (size_t)r + 2]};
    const float dd[3] = {d[3 * (size_t)r], d[3 * (size_t)r + 1], d[3 * (size_t)r + 2]};
    const uint32_t begin = WRITE ? first[j] : 0u;
    uint32_t kept = 0;
    bool dropped = false;
    for (uint32_t base = 0; base < n; base += dg::kWave) {
        const uint32_t s = base + lane;
        const float xi = counter_jitter(seed, r, k, s);
        const float t = t_in + ((float)s + xi) * width;
        float u3[3];
#pragma unroll
        for (int a = 0; a < 3; ++a) {
            const float x = __builtin_fmaf(t, dd[a], oo[a]);
            u3[a] = (x - box.lo[a]) * box.inv_ext[a];
        }
        const bool keep = s < n && bit_of(bits, cell_of(occ, u3));      // empty space is skipped
        const unsigned long long mask = __ballot(keep);
        if (WRITE && keep) {
            const uint32_t pos = begin + kept + (uint32_t)__popcll(mask & ((1ull << lane) - 1ull));
            if (pos < capacity) {
                out.u[3 * (size_t)pos] = u3[0]; out.u[3 * (size_t)pos + 1] = u3[1]; out.u[3 * (size_t)pos + 2] = u3[2];
                out.delta[pos] = width;
                out.t[pos] = t;
                out.sample_ray[pos] = r;
            } else {
                dropped = true;
            }
        }
        kept += (uint32_t)__popcll(mask);
    }
    if (!WRITE && lane == 0) first[j] = kept;
    if (WRITE && dropped) atomicOr(status, 2u);
}

// ---------------------------------------------------------------- exclusive scan of uint32 values, in place
__device__ __forceinline__ uint32_t wave_inclusive(uint32_t v, uint32_t lane)
{
#pragma unroll
    for (int off = 1; off < dg::kWave; off <<= 1) {
        const uint32_t up = __shfl_up(v, off, dg::kWave);
        if (lane >= (uint32_t)off) v += up;
    }
    return v;
}

// exclusive prefix of x over the workgroup (WAVES wavefronts); total receives the sum of all
template <int WAVES>
__device__ __forceinline__ uint32_t block_exclusive(uint32_t x, uint32_t *wave_sums, uint32_t &total)
{
    const uint32_t lane = threadIdx.x % dg::kWave, wave = threadIdx.x / dg::kWave;
    const uint32_t incl = wave_inclusive(x, lane);
    if (lane == dg::kWave - 1) wave_sums[wave] = incl;
    __syncthreads();
    uint32_t before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) {
        const uint32_t v = wave_sums[w];
        before += (uint32_t)w < wave ? v : 0u;
        all += v;
    }
    __syncthreads();                                      // wave_sums may be reused by the caller's next round
    total = all;
    return before + incl - x;
}

__global__ void __launch_bounds__(kBlock)
scan_tile_sums_kernel(const uint32_t *__restrict__ v, uint32_t n, uint32_t *__restrict__ sums)
{
    __shared__ uint32_t wave_sums[kWavesPerBlock];
    const size_t base = (size_t)blockIdx.x * kScanTile + (size_t)threadIdx.x * kScanItems;
    uint32_t mine = 0;
#pragma unroll
    for (int i = 0; i < kScanItems; ++i) mine += base + i < n ? v[base + i] : 0u;
    uint32_t total;
    block_exclusive<kWavesPerBlock>(mine, wave_sums, total);
    if (threadIdx.x == 0) sums[blockIdx.x] = total;
}

__global__ void __launch_bounds__(kSumsBlock)
scan_sums_kernel(uint32_t *__restrict__ sums, uint32_t n_tiles)
{
    __shared__ uint32_t wave_sums[kSumsBlock / dg::kWave];
    uint32_t carry = 0;
    for (uint32_t base = 0; base < n_tiles; base += kSumsBlock) {         // the bound is uniform over the workgroup
        const uint32_t i = base + threadIdx.x;
        const uint32_t x = i < n_tiles ? sums[i] : 0u;
        uint32_t total;
        const uint32_t excl = block_exclusive<kSumsBlock / dg::kWave>(x, wave_sums, total);
        if (i < n_tiles) sums[i] = carry + excl;
        carry += total;
    }
}

__global__ void __launch_bounds__(kBlock)
scan_apply_kernel(uint32_t *__restrict__ v, uint32_t n, const uint32_t *__restrict__ sums)
{
    __shared__ uint32_t wave_sums[kWavesPerBlock];
    const size_t base = (size_t)blockIdx.x * kScanTile + (size_t)threadIdx.x * kScanItems;
    uint32_t x[kScanItems], mine = 0;
#pragma unroll
    for (int i = 0; i < kScanItems; ++i) { x[i] = base + i < n ? v[base + i] : 0u; mine += x[i]; }
    uint32_t total;
    uint32_t run = sums[blockIdx.x] + block_exclusive<kWavesPerBlock>(mine, wave_sums, total);
#pragma unroll
    for (int i = 0; i < kScanItems; ++i) {
        if (base + i < n) v[base + i] = run;
        run += x[i];
    }
}

uint32_t scan_tiles(uint32_t n) { return (uint32_t)(((uint64_t)n + kScanTile - 1) / kScanTile); }

OccArgs occ_args(const dg_occ_desc *desc)
{
    OccArgs g;
    for (int a = 0; a < 3; ++a) { g.res[a] = desc->res[a]; g.scale[a] = desc->scale[a]; }
    g.n_cells = desc->n_cells;
    return g;
}

int occ_desc_ok(const dg_occ_desc *desc, const char *who)
{
    DG_REQUIRE(desc, DG_ERR_ARG, "%s: null descriptor", who);
    DG_REQUIRE(desc->res[0] && desc->res[1] && desc->res[2] &&
                   (uint64_t)desc->res[0] * desc->res[1] * desc->res[2] == desc->n_cells,
               DG_ERR_ARG, "%s: descriptor not initialised by dg_occ_desc_init", who);
    return DG_OK;
}

}  // namespace

extern "C" int dg_occ_desc_init(dg_occ_desc *desc, uint32_t N, const double extent[3])
{
    DG_REQUIRE(desc && extent, DG_ERR_ARG, "dg_occ_desc_init: null pointer");
    DG_REQUIRE(N >= 1, DG_ERR_ARG, "dg_occ_desc_init: resolution must be at least 1");
    DG_REQUIRE(extent[0] > 0 && extent[1] > 0 && extent[2] > 0, DG_ERR_ARG, "dg_occ_desc_init: box extents must be positive");
    std::memset(desc, 0, sizeof *desc);
    const double longest = std::fmax(extent[0], std::fmax(extent[1], extent[2]));
    uint64_t cells = 1;
    for (int a = 0; a < 3; ++a) {
        const double along = extent[a] / longest * (double)N;       // the hash grid's rule at one resolution (Sec. 4.1)
        const uint32_t r = (uint32_t)std::ceil(along);
        desc->res[a] = r ? r : 1u;
        desc->scale[a] = (float)along;
        cells *= desc->res[a];
        DG_REQUIRE(cells <= 0x80000000ull, DG_ERR_UNSUPPORTED, "dg_occ_desc_init: more than 2^31 cells");
    }
    desc->n_cells = (uint32_t)cells;
    return DG_OK;
}

extern "C" void dg_occ_schedule(uint64_t iteration, int *update_now, int *warmup, float *decay, float *threshold)
{
    if (update_now) *update_now = iteration % 16 == 0;
    if (warmup) *warmup = iteration < 4096;
    if (decay) *decay = 0.99f;
    if (threshold) *threshold = iteration < 10000 ? 0.6f : 60.0f;
}

extern "C" int dg_occ_candidates(const dg_occ_desc *desc, const uint32_t *bits, uint32_t i0, uint32_t M, uint32_t n_uniform,
                                 int warmup, uint64_t seed, uint32_t iteration, uint32_t tries, uint32_t *cell, float *u,
                                 void *stream)
{
    if (int rc = occ_desc_ok(desc, "dg_occ_candidates")) return rc;
    DG_REQUIRE((uint64_t)i0 + M <= (1u << 28) && iteration < (1u << 28), DG_ERR_UNSUPPORTED,
               "dg_occ_candidates: candidate indices and iteration must be below 2^28");
    DG_REQUIRE(tries >= 1 && tries <= 64, DG_ERR_ARG, "dg_occ_candidates: tries=%u outside 1..64", tries);
    DG_REQUIRE(!warmup || (uint64_t)i0 + M <= desc->n_cells, DG_ERR_ARG, "dg_occ_candidates: the warm-up rule visits cell i, i0 + M exceeds n_cells");
    if (M == 0) return DG_OK;
    DG_REQUIRE(cell && u && (warmup || n_uniform >= i0 + M || bits), DG_ERR_ARG, "dg_occ_candidates: null pointer");
    candidates_kernel<<<(M + kBlock - 1) / kBlock, kBlock, 0, (hipStream_t)stream>>>(occ_args(desc), bits, i0, M, n_uniform, warmup,
                                                                                    seed, iteration, tries, cell, u);
    return dg::launch_status("dg_occ_candidates");
}

extern "C" int dg_occ_decay(float *density, uint32_t n_cells, float factor, void *stream)
{
    if (n_cells == 0) return DG_OK;
    DG_REQUIRE(density, DG_ERR_ARG, "dg_occ_decay: null pointer");
    const uint32_t n_blocks = (uint32_t)(((uint64_t)n_cells + kBlock - 1) / kBlock);
    decay_kernel<<<n_blocks, kBlock, 0, (hipStream_t)stream>>>(density, n_cells, factor);
    return dg::launch_status("dg_occ_decay");
}

extern "C" int dg_occ_update(float *density, uint32_t n_cells, const uint32_t *cell, const float *sigma, uint32_t M, void *stream)
{
    if (M == 0) return DG_OK;
    DG_REQUIRE(density && cell && sigma, DG_ERR_ARG, "dg_occ_update: null pointer");
    const uint32_t n_blocks = (uint32_t)(((uint64_t)M + kBlock - 1) / kBlock);
    update_kernel<<<n_blocks, kBlock, 0, (hipStream_t)stream>>>(density, n_cells, cell, sigma, M);
    return dg::launch_status("dg_occ_update");
}

extern "C" int dg_occ_bits(const float *density, uint32_t n_cells, float threshold, uint32_t *bits, uint32_t *n_set, void *stream)
{
    if (n_cells == 0) return DG_OK;
    DG_REQUIRE(density && bits, DG_ERR_ARG, "dg_occ_bits: null pointer");
    const uint64_t per_block = (uint64_t)kBlock * kBitsRounds;
    const uint32_t n_blocks = (uint32_t)(((uint64_t)n_cells + per_block - 1) / per_block);
    bits_kernel<<<n_blocks, kBlock, 0, (hipStream_t)stream>>>(density, n_cells, threshold, bits, n_set);
    return dg::launch_status("dg_occ_bits");
}

extern "C" size_t dg_march_workspace_bytes(uint32_t n_seg)
{
    const size_t bytes = (size_t)scan_tiles(n_seg + 1u) * sizeof(uint32_t);      // n_seg < 2^32 - 1 is checked at the call
    return (bytes + 255u) / 256u * 256u;
}

extern "C" int dg_march_segments(const float *o, const float *d, const float *seg_t, const uint32_t *seg_ray,
                                 const uint32_t *seg_slot, uint32_t n_seg, uint32_t k_max, const float *box,
                                 const dg_occ_desc *occ, const uint32_t *bits, float dt, uint32_t max_steps, uint64_t seed,
                                 uint32_t capacity, uint32_t *first, float *u, float *delta, float *t, uint32_t *sample_ray,
                                 uint32_t *status, void *ws, size_t ws_bytes, void *stream)
{
    if (int rc = occ_desc_ok(occ, "dg_march_segments")) return rc;
    DG_REQUIRE(box && k_max >= 1 && dt > 0.0f && max_steps >= 1 && max_steps <= 65535, DG_ERR_ARG,
               "dg_march_segments: bad box, k_max, dt or max_steps (1..65535)");
    DG_REQUIRE(n_seg < 0xffffffffu, DG_ERR_UNSUPPORTED, "dg_march_segments: too many segments");
    DG_REQUIRE(first && status && ws, DG_ERR_ARG, "dg_march_segments: null pointer");
    DG_REQUIRE(ws_bytes >= dg_march_workspace_bytes(n_seg), DG_ERR_WORKSPACE, "dg_march_segments: workspace of %zu bytes, %zu needed",
               ws_bytes, dg_march_workspace_bytes(n_seg));
    DG_REQUIRE(n_seg == 0 || (o && d && seg_t && seg_ray && seg_slot && bits), DG_ERR_ARG, "dg_march_segments: null pointer");
    DG_REQUIRE(capacity == 0 || (u && delta && t && sample_ray), DG_ERR_ARG, "dg_march_segments: null output");
    BoxArgs b;
    for (int a = 0; a < 3; ++a) {
        DG_REQUIRE(box[3 + a] > box[a], DG_ERR_ARG, "dg_march_segments: empty box");
        b.lo[a] = box[a];
        b.inv_ext[a] = 1.0f / (box[3 + a] - box[a]);
    }
    hipStream_t st = (hipStream_t)stream;
    const OccArgs g = occ_args(occ);
    const MarchOut out = {u, delta, t, sample_ray};
    const uint32_t seg_blocks = n_seg ? (n_seg + kWavesPerBlock - 1) / kWavesPerBlock : 1u;
    uint32_t *sums = (uint32_t *)ws;
    const uint32_t n_vals = n_seg + 1u, n_tiles = scan_tiles(n_vals);
    march_kernel<false><<<seg_blocks, kBlock, 0, st>>>(o, d, seg_t, seg_ray, seg_slot, n_seg, k_max, b, g, bits, dt, max_steps, seed,
                                                       capacity, first, out, status);
    scan_tile_sums_kernel<<<n_tiles, kBlock, 0, st>>>(first, n_vals, sums);
    scan_sums_kernel<<<1, kSumsBlock, 0, st>>>(sums, n_tiles);
    scan_apply_kernel<<<n_tiles, kBlock, 0, st>>>(first, n_vals, sums);
    if (n_seg)
        march_kernel<true><<<seg_blocks, kBlock, 0, st>>>(o, d, seg_t, seg_ray, seg_slot, n_seg, k_max, b, g, bits, dt, max_steps,
                                                          seed, capacity, first, out, status);
    return dg::launch_status("dg_march_segments");
}
