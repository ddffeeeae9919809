// Ray / box segments, distribution to partitions, stratified sampling, direction encoding
// (Sec. 4.2.1, Sec. 4.4.2, Fig. 2 steps 2-3).  All of it is light streaming work: one thread
// per ray or per sample, coalesced where the layout allows.
//
// The fp32 bookkeeping here must round after every operation (segment times are compared bit
// for bit between boxes), so this file is built with -ffp-contract=off.
#include "dg_internal.h"
#include "sample_common.h"
#include <mutex>

#pragma clang fp contract(off)

namespace {

constexpr int kBlock = 256;
constexpr uint32_t kMaxK = 12;

// ---------------------------------------------------------------- ray / box slab test
// interval of the ray inside one box, clipped to t >= t_min; false = miss
__device__ __forceinline__ bool slab_interval(const float (&oo)[3], const float (&dd)[3], const float (&inv)[3], const float *lo,
                                              const float *hi, float t_min, float &t_in, float &t_out)
{
    float tn = -INFINITY, tf = INFINITY;
    bool miss = false;
    for (int a = 0; a < 3; ++a) {
        if (dd[a] == 0.0f) {
            if (!(lo[a] <= oo[a] && oo[a] < hi[a])) miss = true;   // half-open: shared faces go up
            continue;
        }
        const float t1 = (lo[a] - oo[a]) * inv[a];
        const float t2 = (hi[a] - oo[a]) * inv[a];
        tn = fmaxf(tn, fminf(t1, t2));
        tf = fminf(tf, fmaxf(t1, t2));
    }
    t_in = fmaxf(tn, t_min);
    t_out = tf;
    return !miss && t_out > t_in;
}

struct SegmentList {
    float tin[kMaxK], tout[kMaxK];
    int32_t pid[kMaxK];
    uint32_t cnt;
    bool overflow;
};

// sorted insert, front to back; equal entry times keep the order of insertion
__device__ __forceinline__ void insert_segment(SegmentList &L, uint32_t k_max, float t_in, float t_out, int32_t p)
{
    uint32_t pos = L.cnt;
    while (pos > 0 && L.tin[pos - 1] > t_in) --pos;
    if (L.cnt >= k_max) L.overflow = true;
    if (pos >= k_max) return;
    const uint32_t last = L.cnt < k_max ? L.cnt : k_max - 1;
    for (uint32_t k = last; k > pos; --k) { L.tin[k] = L.tin[k - 1]; L.tout[k] = L.tout[k - 1]; L.pid[k] = L.pid[k - 1]; }
    L.tin[pos] = t_in; L.tout[pos] = t_out; L.pid[pos] = p;
    if (L.cnt < k_max) ++L.cnt;
}

// A partition covers its box minus its hole (Sec. 4.2.2: coarse sub-models cover the outer box around the inner one);
// a ray meets such a region in up to two pieces, [t_in, hole entry] and [hole exit, t_out].
__global__ void __launch_bounds__(kBlock)
ray_aabb_kernel(const float *__restrict__ o, const float *__restrict__ d, uint32_t R,
                const float *__restrict__ parts, const float *__restrict__ holes, uint32_t P, float t_min, uint32_t k_max,
                uint32_t *__restrict__ seg_count, float *__restrict__ seg_t, int32_t *__restrict__ seg_part,
                uint32_t *__restrict__ status)
{
    __shared__ float boxes[DG_MAX_PARTITIONS * 6], hboxes[DG_MAX_PARTITIONS * 6];
    for (uint32_t i = threadIdx.x; i < P * 6; i += kBlock) { boxes[i] = parts[i]; hboxes[i] = holes ? holes[i] : 0.0f; }
    __syncthreads();
    const uint32_t r = blockIdx.x * kBlock + threadIdx.x;
    if (r >= R) return;
    const float oo[3] = {o[3 * r], o[3 * r + 1], o[3 * r + 2]}, dd[3] = {d[3 * r], d[3 * r + 1], d[3 * r + 2]};
    float inv[3];
    for (int a = 0; a < 3; ++a) inv[a] = dd[a] != 0.0f ? 1.0f / dd[a] : 0.0f;

    SegmentList L;
    L.cnt = 0;
    L.overflow = false;
    for (uint32_t p = 0; p < P; ++p) {
        const float *lo = boxes + 6 * p, *hi = lo + 3, *hlo = hboxes + 6 * p, *hhi = hlo + 3;
        float t_in, t_out, h_in, h_out;
        if (!slab_interval(oo, dd, inv, lo, hi, t_min, t_in, t_out)) continue;
        const bool has_hole = hhi[0] > hlo[0] && hhi[1] > hlo[1] && hhi[2] > hlo[2];      // a hole with no volume is no hole
        if (has_hole && slab_interval(oo, dd, inv, hlo, hhi, t_min, h_in, h_out)) {
            // a hole may overhang its box: the pieces are cut to the box's own interval
            const float first_end = fminf(h_in, t_out), second_begin = fmaxf(h_out, t_in);
            if (first_end > t_in) insert_segment(L, k_max, t_in, first_end, (int32_t)p);
            if (t_out > second_begin) insert_segment(L, k_max, second_begin, t_out, (int32_t)p);
        } else {
            insert_segment(L, k_max, t_in, t_out, (int32_t)p);
        }
    }
    seg_count[r] = L.cnt;
    for (uint32_t k = 0; k < k_max; ++k) {
        const bool used = k < L.cnt;
        seg_t[((size_t)r * k_max + k) * 2] = used ? L.tin[k] : 0.0f;
        seg_t[((size_t)r * k_max + k) * 2 + 1] = used ? L.tout[k] : 0.0f;
        seg_part[(size_t)r * k_max + k] = used ? L.pid[k] : -1;
    }
    if (L.overflow) atomicOr(status, 1u);
}

// ---------------------------------------------------------------- stable distribution to boxes
// Three passes: per-block histogram, scan over blocks, scatter with in-block stable ranks.
// A ray holds at most two segments per partition (a convex box is crossed once; a box with a hole in up to two pieces).
__global__ void __launch_bounds__(kBlock)
bucket_count_kernel(const uint32_t *__restrict__ seg_count, const int32_t *__restrict__ seg_part, uint32_t R,
                    uint32_t k_max, uint32_t P, uint32_t n_blocks, uint32_t *__restrict__ block_hist)
{
    __shared__ uint32_t hist[DG_MAX_PARTITIONS];
    if (threadIdx.x < DG_MAX_PARTITIONS) hist[threadIdx.x] = 0;
    __syncthreads();
    const uint32_t r = blockIdx.x * kBlock + threadIdx.x;
    if (r < R) {
        const uint32_t cnt = seg_count[r];
        for (uint32_t k = 0; k < cnt; ++k) atomicAdd(&hist[seg_part[(size_t)r * k_max + k]], 1u);
    }
    __syncthreads();
    if (threadIdx.x < P) block_hist[(size_t)threadIdx.x * n_blocks + blockIdx.x] = hist[threadIdx.x];
}

// one wavefront per box at a time: exclusive scan of that box's per-block counts; then box offsets
constexpr int kScanThreads = 1024;
__global__ void __launch_bounds__(kScanThreads)
bucket_scan_kernel(uint32_t P, uint32_t n_blocks, uint32_t *__restrict__ block_hist, uint32_t *__restrict__ part_offset)
{
    __shared__ uint32_t totals[DG_MAX_PARTITIONS];
    const uint32_t wave = threadIdx.x / dg::kWave, lane = threadIdx.x % dg::kWave;
    for (uint32_t p = wave; p < P; p += kScanThreads / dg::kWave) {
        uint32_t *row = block_hist + (size_t)p * n_blocks;
        uint32_t carry = 0;
        for (uint32_t base = 0; base < n_blocks; base += dg::kWave) {
            const uint32_t i = base + lane;
            const uint32_t v = i < n_blocks ? row[i] : 0u;
            uint32_t incl = v;
            for (int off = 1; off < dg::kWave; off <<= 1) {
                const uint32_t up = __shfl_up(incl, off, dg::kWave);
                if ((int)lane >= off) incl += up;
            }
            if (i < n_blocks) row[i] = carry + incl - v;
            carry += __shfl(incl, dg::kWave - 1, dg::kWave);
        }
        if (lane == 0) totals[p] = carry;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t run = 0;
        for (uint32_t q = 0; q < P; ++q) { part_offset[q] = run; run += totals[q]; }
        part_offset[P] = run;
    }
}

__global__ void __launch_bounds__(kBlock)
bucket_scatter_kernel(const uint32_t *__restrict__ seg_count, const int32_t *__restrict__ seg_part, uint32_t R,
                      uint32_t k_max, uint32_t P, uint32_t n_blocks, const uint32_t *__restrict__ block_hist,
                      const uint32_t *__restrict__ part_offset, uint32_t *__restrict__ seg_ray,
                      uint32_t *__restrict__ seg_slot)
{
    constexpr int kWaves = kBlock / dg::kWave;
    __shared__ uint32_t wave_count[kWaves];
    const uint32_t r = blockIdx.x * kBlock + threadIdx.x;
    const uint32_t lane = threadIdx.x % dg::kWave, wave = threadIdx.x / dg::kWave;
    uint32_t cnt = 0;
    int32_t mine[kMaxK];
    if (r < R) {
        cnt = seg_count[r];
        for (uint32_t k = 0; k < kMaxK; ++k) mine[k] = (k < cnt && k < k_max) ? seg_part[(size_t)r * k_max + k] : -1;
    }
    for (uint32_t p = 0; p < P; ++p) {
        int first = -1, second = -1;          // this ray's slots in box p, front to back
        for (uint32_t k = 0; k < kMaxK; ++k)
            if (k < cnt && mine[k] == (int32_t)p) { if (first < 0) first = (int)k; else second = (int)k; }
        const unsigned long long vote1 = __ballot(first >= 0), vote2 = __ballot(second >= 0);
        const unsigned long long below = (1ull << lane) - 1ull;
        const uint32_t before = __popcll(vote1 & below) + __popcll(vote2 & below);
        if (lane == 0) wave_count[wave] = __popcll(vote1) + __popcll(vote2);
        __syncthreads();
        uint32_t base = 0;
        for (uint32_t w = 0; w < wave; ++w) base += wave_count[w];
        __syncthreads();
        if (first >= 0) {
            const uint32_t dst = part_offset[p] + block_hist[(size_t)p * n_blocks + blockIdx.x] + base + before;
            seg_ray[dst] = r;
            seg_slot[dst] = (uint32_t)first;
            if (second >= 0) { seg_ray[dst + 1] = r; seg_slot[dst + 1] = (uint32_t)second; }
        }
    }
}

// ---------------------------------------------------------------- stratified samples
using dg_sample::counter_jitter;
using dg_sample::BoxArgs;

__global__ void __launch_bounds__(kBlock)
sample_kernel(const float *__restrict__ o, const float *__restrict__ d, const float *__restrict__ seg_t,
              const uint32_t *__restrict__ seg_ray, const uint32_t *__restrict__ seg_slot, uint64_t n_samples,
              uint32_t k_max, BoxArgs box, uint32_t S, uint64_t seed, const float *__restrict__ jitter,
              float *__restrict__ u, float *__restrict__ delta, float *__restrict__ t_samples)
{
    const uint64_t n = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (n >= n_samples) return;
    const uint32_t j = (uint32_t)(n / S), s = (uint32_t)(n % S);
    const uint32_t r = seg_ray[j], k = seg_slot[j];
    const float t_in = seg_t[((size_t)r * k_max + k) * 2], t_out = seg_t[((size_t)r * k_max + k) * 2 + 1];
    const float dt = (t_out - t_in) / (float)S;
    const float xi = jitter ? jitter[n] : counter_jitter(seed, r, k, s);
    const float t = t_in + ((float)s + xi) * dt;
    for (int a = 0; a < 3; ++a) {
        const float x = __builtin_fmaf(t, d[3 * r + a], o[3 * r + a]);
        u[3 * n + a] = (x - box.lo[a]) * box.inv_ext[a];
    }
    delta[n] = dt;
    if (t_samples) t_samples[n] = t;
}

// ---------------------------------------------------------------- real spherical harmonics
// Cartesian forms of Y_l^m for l <= 3 on the unit vector, Condon-Shortley phase included.
__global__ void __launch_bounds__(kBlock)
dir_encode_kernel(const float *__restrict__ d, const uint32_t *__restrict__ index, uint64_t n, uint32_t degree,
                  __half *__restrict__ out)
{
    const uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= n) return;
    const size_t r = index ? index[i] : i;
    float x = d[3 * r], y = d[3 * r + 1], z = d[3 * r + 2];
    const float len = sqrtf(x * x + y * y + z * z);
    if (len > 0.0f) { const float q = 1.0f / len; x *= q; y *= q; z *= q; } else { x = 0.0f; y = 0.0f; z = 1.0f; }
    float v[16];
    v[0] = 0.28209479177387814f;
    v[1] = -0.4886025119029199f * y;
    v[2] = 0.4886025119029199f * z;
    v[3] = -0.4886025119029199f * x;
    const float xx = x * x, yy = y * y, zz = z * z;
    v[4] = 1.0925484305920792f * x * y;
    v[5] = -1.0925484305920792f * y * z;
    v[6] = 0.31539156525252005f * (3.0f * zz - 1.0f);
    v[7] = -1.0925484305920792f * x * z;
    v[8] = 0.5462742152960396f * (xx - yy);
    v[9] = -0.5900435899266435f * y * (3.0f * xx - yy);
    v[10] = 2.890611442640554f * x * y * z;
    v[11] = -0.4570457994644658f * y * (5.0f * zz - 1.0f);
    v[12] = 0.3731763325901154f * z * (5.0f * zz - 3.0f);
    v[13] = -0.4570457994644658f * x * (5.0f * zz - 1.0f);
    v[14] = 1.445305721320277f * z * (xx - yy);
    v[15] = -0.5900435899266435f * x * (xx - 3.0f * yy);
    const uint32_t nd = degree * degree;
    if (degree == 4 && (reinterpret_cast<uintptr_t>(out) & 15u) == 0) {
        // the full row as two 16-byte stores (a loop over a run-time count would index v[] through memory)
        __half2 h[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) h[k] = __floats2half2_rn(v[2 * k], v[2 * k + 1]);
        uint4 *dst = reinterpret_cast<uint4 *>(out + i * 16);
        dst[0] = *reinterpret_cast<const uint4 *>(&h[0]);
        dst[1] = *reinterpret_cast<const uint4 *>(&h[4]);
        return;
    }
#pragma unroll
    for (uint32_t k = 0; k < 16; ++k)
        if (k < nd) out[i * nd + k] = __float2half_rn(v[k]);
}

// appearance rows (Sec. 4.4.3): one 16-byte piece of a row per thread
__global__ void __launch_bounds__(kBlock)
appearance_rows_kernel(const uint4 *__restrict__ table, const uint32_t *__restrict__ image_of_ray, const uint32_t *__restrict__ index,
                       uint64_t n, uint32_t pieces, uint4 *__restrict__ out)
{
    const uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i >= n * pieces) return;
    const uint64_t row = i / pieces;
    const uint32_t piece = (uint32_t)(i % pieces);
    const size_t ray = index ? index[row] : row;
    out[i] = table[(size_t)image_of_ray[ray] * pieces + piece];
}

}  // namespace

extern "C" size_t dg_segments_workspace_bytes(uint32_t R, uint32_t P)
{
    const size_t n_blocks = ((size_t)R + kBlock - 1) / kBlock;
    return (n_blocks ? n_blocks : 1) * (size_t)P * sizeof(uint32_t);
}

namespace {

// shared by the two entry points below: argument checks and the four launches; hist is the [P, n_blocks] counter table
int ray_aabb_segments(const char *who, const float *o, const float *d, uint32_t R, const float *parts, const float *holes,
                      uint32_t P, float t_min, uint32_t k_max, uint32_t *seg_count, float *seg_t, int32_t *seg_part,
                      uint32_t *part_offset, uint32_t *seg_ray, uint32_t *seg_slot, uint32_t *status, uint32_t *hist,
                      hipStream_t st)
{
    const uint32_t n_blocks = (R + kBlock - 1) / kBlock;
    if (R > 0) {
        ray_aabb_kernel<<<n_blocks, kBlock, 0, st>>>(o, d, R, parts, holes, P, t_min, k_max, seg_count, seg_t, seg_part, status);
    }
    if (part_offset) {
        if (R > 0)
            bucket_count_kernel<<<n_blocks, kBlock, 0, st>>>(seg_count, seg_part, R, k_max, P, n_blocks, hist);
        bucket_scan_kernel<<<1, kScanThreads, 0, st>>>(P, n_blocks, hist, part_offset);
        if (R > 0)
            bucket_scatter_kernel<<<n_blocks, kBlock, 0, st>>>(seg_count, seg_part, R, k_max, P, n_blocks, hist,
                                                               part_offset, seg_ray, seg_slot);
    }
    return dg::launch_status(who);
}

int check_segment_args(const char *who, const float *o, const float *d, uint32_t R, const float *parts, uint32_t P, uint32_t k_max,
                       const uint32_t *seg_count, const float *seg_t, const int32_t *seg_part, const uint32_t *part_offset,
                       const uint32_t *seg_ray, const uint32_t *seg_slot, const uint32_t *status)
{
    DG_REQUIRE(P >= 1 && P <= DG_MAX_PARTITIONS, DG_ERR_UNSUPPORTED, "%s: P=%u outside 1..%d", who, P, DG_MAX_PARTITIONS);
    DG_REQUIRE(k_max >= 1 && k_max <= kMaxK, DG_ERR_UNSUPPORTED, "%s: k_max=%u outside 1..%u", who, k_max, kMaxK);
    DG_REQUIRE(parts && status, DG_ERR_ARG, "%s: null parts/status", who);
    DG_REQUIRE(R == 0 || (o && d && seg_count && seg_t && seg_part), DG_ERR_ARG, "%s: null ray or output pointer", who);
    DG_REQUIRE(!part_offset || R == 0 || (seg_ray && seg_slot), DG_ERR_ARG, "%s: part_offset given without seg_ray/seg_slot", who);
    return DG_OK;
}

}  // namespace

extern "C" int dg_ray_aabb_segments(const float *o, const float *d, uint32_t R, const float *parts, const float *holes,
                                    uint32_t P, float t_min, uint32_t k_max, uint32_t *seg_count, float *seg_t,
                                    int32_t *seg_part, uint32_t *part_offset, uint32_t *seg_ray,
                                    uint32_t *seg_slot, uint32_t *status, void *ws, size_t ws_bytes, void *stream)
{
    const char *who = "dg_ray_aabb_segments";
    if (int rc = check_segment_args(who, o, d, R, parts, P, k_max, seg_count, seg_t, seg_part, part_offset, seg_ray, seg_slot, status)) return rc;
    if (part_offset)
        DG_REQUIRE(ws && ws_bytes >= dg_segments_workspace_bytes(R, P), DG_ERR_WORKSPACE,
                   "dg_ray_aabb_segments: workspace %zu < %zu bytes", ws_bytes, dg_segments_workspace_bytes(R, P));
    return ray_aabb_segments(who, o, d, R, parts, holes, P, t_min, k_max, seg_count, seg_t, seg_part, part_offset, seg_ray, seg_slot,
                             status, (uint32_t *)ws, (hipStream_t)stream);
}

// ---------------------------------------------------------------- the same call for callers that cannot allocate
// The counter table of the distribution step lives in a fixed device array instead of a caller's workspace.
constexpr size_t kStaticCounters = DG_SEGMENTS_STATIC_COUNTERS;        // 1 MiB: R/256 blocks x P boxes, e.g. 2^20 rays x 64 boxes
static __device__ __align__(256) uint32_t scratch[kStaticCounters];   // one copy per GPU, held until the process ends

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_lock;
uint32_t *g_scratch_ptr[kMaxDevices] = {};     // device address of `scratch` on each GPU, looked up once per device

// `scratch` as host code sees it is only a handle: the address kernels can use comes from the runtime, per device
int static_counters(uint32_t **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return dg::fail(DG_ERR_HIP, "dg_ray_aabb_segments_static: hipGetDevice: %s", hipGetErrorString(e));
    DG_REQUIRE(dev >= 0 && dev < kMaxDevices, DG_ERR_UNSUPPORTED, "dg_ray_aabb_segments_static: device %d outside 0..%d", dev, kMaxDevices - 1);
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return dg::fail(DG_ERR_HIP, "dg_ray_aabb_segments_static: hipGetSymbolAddress: %s", hipGetErrorString(e));
        g_scratch_ptr[dev] = (uint32_t *)p;
    }
    *out = g_scratch_ptr[dev];
    return DG_OK;
}
}  // namespace

extern "C" int dg_ray_aabb_segments_static(const float *o, const float *d, uint32_t R, const float *parts, const float *holes,
                                           uint32_t P, float t_min, uint32_t k_max, uint32_t *seg_count, float *seg_t,
                                           int32_t *seg_part, uint32_t *part_offset, uint32_t *seg_ray, uint32_t *seg_slot,
                                           uint32_t *status, void *stream)
{
    const char *who = "dg_ray_aabb_segments_static";
    if (int rc = check_segment_args(who, o, d, R, parts, P, k_max, seg_count, seg_t, seg_part, part_offset, seg_ray, seg_slot, status)) return rc;
    const size_t counters = dg_segments_workspace_bytes(R, P) / sizeof(uint32_t);
    DG_REQUIRE(counters <= kStaticCounters, DG_ERR_WORKSPACE,
               "dg_ray_aabb_segments_static: ceil(R/256) * P = %zu counters exceed the fixed table of %zu (R=%u, P=%u); use "
               "dg_ray_aabb_segments with a workspace", counters, kStaticCounters, R, P);
    uint32_t *hist = nullptr;
    if (int rc = static_counters(&hist)) return rc;
    // nothing to clear: the counting kernel writes every counter [p < P, block < ceil(R/256)] the later kernels read
    return ray_aabb_segments(who, o, d, R, parts, holes, P, t_min, k_max, seg_count, seg_t, seg_part, part_offset, seg_ray, seg_slot,
                             status, hist, (hipStream_t)stream);
}

extern "C" int dg_sample_segments(const float *o, const float *d, const float *seg_t, const uint32_t *seg_ray,
                                  const uint32_t *seg_slot, uint32_t n_seg, uint32_t k_max, const float *box,
                                  uint32_t S, uint64_t seed, const float *jitter, float *u, float *delta,
                                  float *t_samples, void *stream)
{
    DG_REQUIRE(box && S >= 1 && S <= 65535 && k_max >= 1, DG_ERR_ARG, "dg_sample_segments: bad box/S/k_max");
    if (n_seg == 0) return DG_OK;
    DG_REQUIRE(o && d && seg_t && seg_ray && seg_slot && u && delta, DG_ERR_ARG, "dg_sample_segments: null pointer");
    BoxArgs b;
    for (int a = 0; a < 3; ++a) {
        DG_REQUIRE(box[3 + a] > box[a], DG_ERR_ARG, "dg_sample_segments: empty box");
        b.lo[a] = box[a];
        b.inv_ext[a] = 1.0f / (box[3 + a] - box[a]);
    }
    const uint64_t n = (uint64_t)n_seg * S;
    const uint64_t n_blocks = (n + kBlock - 1) / kBlock;
    DG_REQUIRE(n_blocks <= 0x7fffffffull, DG_ERR_UNSUPPORTED, "dg_sample_segments: too many samples");
    sample_kernel<<<(uint32_t)n_blocks, kBlock, 0, (hipStream_t)stream>>>(o, d, seg_t, seg_ray, seg_slot, n, k_max, b, S,
                                                                          seed, jitter, u, delta, t_samples);
    return dg::launch_status("dg_sample_segments");
}

extern "C" int dg_dir_encode(const float *d, const uint32_t *index, uint64_t n, uint32_t degree, void *out,
                             void *stream)
{
    DG_REQUIRE(degree >= 1 && degree <= 4, DG_ERR_UNSUPPORTED, "dg_dir_encode: degree %u outside 1..4", degree);
    if (n == 0) return DG_OK;
    DG_REQUIRE(d && out, DG_ERR_ARG, "dg_dir_encode: null pointer");
    const uint64_t n_blocks = (n + kBlock - 1) / kBlock;
    DG_REQUIRE(n_blocks <= 0x7fffffffull, DG_ERR_UNSUPPORTED, "dg_dir_encode: too many rows");
    dir_encode_kernel<<<(uint32_t)n_blocks, kBlock, 0, (hipStream_t)stream>>>(d, index, n, degree, (__half *)out);
    return dg::launch_status("dg_dir_encode");
}

extern "C" int dg_appearance_rows(const void *table, const uint32_t *image_of_ray, const uint32_t *index, uint64_t n,
                                  uint32_t n_app, void *out, void *stream)
{
    DG_REQUIRE(n_app >= 8 && n_app % 8 == 0, DG_ERR_ARG, "dg_appearance_rows: n_app=%u is not a positive multiple of 8", n_app);
    if (n == 0) return DG_OK;
    DG_REQUIRE(table && image_of_ray && out, DG_ERR_ARG, "dg_appearance_rows: null pointer");
    DG_REQUIRE(dg::aligned(table, 16) && dg::aligned(out, 16), DG_ERR_ARG, "dg_appearance_rows: table and out must be 16-byte aligned");
    const uint32_t pieces = n_app / 8;
    const uint64_t n_blocks = (n * pieces + kBlock - 1) / kBlock;
    DG_REQUIRE(n_blocks <= 0x7fffffffull, DG_ERR_UNSUPPORTED, "dg_appearance_rows: too many rows");
    appearance_rows_kernel<<<(uint32_t)n_blocks, kBlock, 0, (hipStream_t)stream>>>((const uint4 *)table, image_of_ray, index, n, pieces,
                                                                                   (uint4 *)out);
    return dg::launch_status("dg_appearance_rows");
}
