// Measured peaks of the MI355X for the access patterns of the hot path: what the chip sustains for a plain stream
// copy, for random 8- and 16-byte gathers out of a table (the hash-grid encode's forward), for random fp32 atomic adds
// (its backward without binning) and for a loop of v_mfma_f32_32x32x16_f16 (the field MLPs).  These are yardsticks for
// the benchmark, kept apart from the library proper (libdgpeaks.so, symbols pk_*): each kernel does nothing but the
// access pattern, with many independent requests in flight per lane, so its rate is an upper bound for any kernel
// that has the same pattern plus arithmetic.
//
// Conventions as in distgrid.h: device pointers owned by the caller, work enqueued on the caller's stream, int return
// (0 ok, -1 bad argument, -4 launch failure); nothing is allocated here.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <cstdint>

namespace {

constexpr int kBlock = 256;
constexpr int kFlight = 8;          // independent requests per lane and loop trip

// 32-bit integer mixer (two multiply-xorshift rounds): consecutive counters -> uncorrelated table positions
__device__ __forceinline__ uint32_t mix32(uint32_t x)
{
    x ^= x >> 16; x *= 0x7feb352du;
    x ^= x >> 15; x *= 0x846ca68bu;
    x ^= x >> 16;
    return x;
}

typedef uint32_t word4 __attribute__((ext_vector_type(4)));
constexpr int kCopyGrid = 256 * 64, kReadGrid = 256 * 32;

// Streams use non-temporal loads and stores: data touched once moves faster past the caches (measured on this chip with
// 4 GiB: copy 4.5 TB/s plain, 5.0 non-temporal; read-only 5.5 plain, 6.2 non-temporal).
__global__ void __launch_bounds__(kBlock) copy_kernel(const word4 *__restrict__ src, word4 *__restrict__ dst, size_t n)
{
    const size_t stride = (size_t)gridDim.x * kBlock;
    for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += stride)
        __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// read-only stream, kFlight loads in flight per lane; the xor of everything read goes to sink[thread]
__global__ void __launch_bounds__(kBlock) read_kernel(const word4 *__restrict__ src, size_t n, uint32_t *__restrict__ sink)
{
    const size_t stride = (size_t)gridDim.x * kBlock;
    size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x;
    uint32_t acc = 0;
    for (; i + (kFlight - 1) * stride < n; i += kFlight * stride) {
        word4 v[kFlight];
#pragma unroll
        for (int k = 0; k < kFlight; ++k) v[k] = __builtin_nontemporal_load(src + i + k * stride);
#pragma unroll
        for (int k = 0; k < kFlight; ++k) acc ^= v[k].x ^ v[k].y ^ v[k].z ^ v[k].w;
    }
    for (; i < n; i += stride) { const word4 a = src[i]; acc ^= a.x ^ a.y ^ a.z ^ a.w; }
    sink[blockIdx.x * kBlock + threadIdx.x] = acc;
}

// every lane reads `per_lane` random entries of the table (T a power of two), kFlight at a time; the xor of everything
// read goes to sink[thread] so that no load can be dropped
template <typename E>
__global__ void __launch_bounds__(kBlock)
gather_kernel(const E *__restrict__ table, uint32_t mask, uint32_t per_lane, uint32_t seed, uint32_t *__restrict__ sink)
{
    const uint32_t t = blockIdx.x * kBlock + threadIdx.x;
    uint32_t acc = 0, ctr = t * per_lane + seed;
    for (uint32_t i = 0; i < per_lane; i += kFlight) {
        E v[kFlight];
#pragma unroll
        for (int k = 0; k < kFlight; ++k) v[k] = table[mix32(ctr + i + k) & mask];
#pragma unroll
        for (int k = 0; k < kFlight; ++k) acc ^= v[k].x ^ v[k].y;
    }
    sink[t] = acc;
}

// every lane adds 1 to `per_lane` random floats of the table, without waiting for a result
__global__ void __launch_bounds__(kBlock)
atomic_kernel(float *__restrict__ table, uint32_t mask, uint32_t per_lane, uint32_t seed)
{
    const uint32_t t = blockIdx.x * kBlock + threadIdx.x;
    const uint32_t ctr = t * per_lane + seed;
    for (uint32_t i = 0; i < per_lane; ++i) unsafeAtomicAdd(table + (mix32(ctr + i) & mask), 1.0f);
}

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));

// four independent accumulator tiles per wavefront, `iters` rounds of four matrix instructions
__global__ void __launch_bounds__(kBlock) mfma_kernel(uint32_t iters, float *__restrict__ sink)
{
    const int lane = threadIdx.x % 64;
    half8 a, b;
#pragma unroll
    for (int j = 0; j < 8; ++j) { a[j] = (_Float16)(0.001f * (float)((lane + j) % 7)); b[j] = (_Float16)(0.002f * (float)((lane * 3 + j) % 5)); }
    float16v c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
    for (uint32_t i = 0; i < iters; ++i) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c3, 0, 0, 0);
    }
    float s = 0.0f;
#pragma unroll
    for (int r = 0; r < 16; ++r) s += c0[r] + c1[r] + c2[r] + c3[r];
    sink[blockIdx.x * kBlock + threadIdx.x] = s;
}

int status()
{
    return hipGetLastError() == hipSuccess ? 0 : -4;
}

}  // namespace

// dst[0, bytes) = src[0, bytes); bytes a multiple of 16, both 16-byte aligned.  Moves 2 * bytes.
extern "C" int pk_stream_copy(const void *src, void *dst, size_t bytes, void *stream)
{
    if (!src || !dst || bytes % 16 || ((uintptr_t)src | (uintptr_t)dst) % 16) return -1;
    if (bytes == 0) return 0;
    copy_kernel<<<kCopyGrid, kBlock, 0, (hipStream_t)stream>>>((const word4 *)src, (word4 *)dst, bytes / 16);
    return status();
}

// reads src[0, bytes) once; sink: 256 * 8192 words (one per lane of the launch).  Moves `bytes`.
extern "C" int pk_stream_read(const void *src, size_t bytes, uint32_t *sink, void *stream)
{
    if (!src || !sink || bytes % 16 || (uintptr_t)src % 16) return -1;
    if (bytes == 0) return 0;
    read_kernel<<<kReadGrid, kBlock, 0, (hipStream_t)stream>>>((const word4 *)src, bytes / 16, sink);
    return status();
}

// n_lanes lanes (a multiple of 256) each read per_lane (a multiple of 8) random entries of entry_bytes (8 or 16) bytes
// out of a table of 2^log2_entries entries; sink: n_lanes words.  n_lanes * per_lane gathers in all (below 2^32).
extern "C" int pk_random_gather(const void *table, uint32_t log2_entries, uint32_t entry_bytes, uint32_t n_lanes, uint32_t per_lane,
                                uint32_t seed, uint32_t *sink, void *stream)
{
    if (!table || !sink || log2_entries > 31 || n_lanes % kBlock || per_lane % kFlight || (entry_bytes != 8 && entry_bytes != 16)) return -1;
    if ((uint64_t)n_lanes * per_lane >= (1ull << 32) || (uintptr_t)table % entry_bytes) return -1;
    if (n_lanes == 0 || per_lane == 0) return 0;
    const uint32_t mask = (1u << log2_entries) - 1u;
    if (entry_bytes == 16)
        gather_kernel<uint4><<<n_lanes / kBlock, kBlock, 0, (hipStream_t)stream>>>((const uint4 *)table, mask, per_lane, seed, sink);
    else
        gather_kernel<uint2><<<n_lanes / kBlock, kBlock, 0, (hipStream_t)stream>>>((const uint2 *)table, mask, per_lane, seed, sink);
    return status();
}

// n_lanes lanes (a multiple of 256) each add 1.0f to per_lane random floats of a table of 2^log2_entries floats
// (fire-and-forget atomics, as a plain scatter-add of the table gradient would issue them)
extern "C" int pk_random_atomic_add(float *table, uint32_t log2_entries, uint32_t n_lanes, uint32_t per_lane, uint32_t seed, void *stream)
{
    if (!table || log2_entries > 31 || n_lanes % kBlock || (uint64_t)n_lanes * per_lane >= (1ull << 32)) return -1;
    if (n_lanes == 0 || per_lane == 0) return 0;
    atomic_kernel<<<n_lanes / kBlock, kBlock, 0, (hipStream_t)stream>>>(table, (1u << log2_entries) - 1u, per_lane, seed);
    return status();
}

// n_waves wavefronts (a multiple of 4) each issue 4 * iters v_mfma_f32_32x32x16_f16 (32768 flop each) on four independent
// accumulators; sink: 64 * n_waves floats
extern "C" int pk_mfma_loop(uint32_t n_waves, uint32_t iters, float *sink, void *stream)
{
    if (!sink || n_waves % 4) return -1;
    if (n_waves == 0) return 0;
    mfma_kernel<<<n_waves / 4, kBlock, 0, (hipStream_t)stream>>>(iters, sink);
    return status();
}
