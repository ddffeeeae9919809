// Hash-grid encode backward without global atomics in the inner loop (Sec. 3.2: the transpose of the
// encode).
//
// Global fp32 atomics on MI355X retire at a fixed rate per distinct cache line an instruction touches
// (about 21 G lines/s measured, whatever the scope or table size), far below what the 8 x N x L
// scattered adds of this pass need.  LDS atomics do not have that limit.  So the table gradient is
// built by binning:
//   * levels whose tables fit LDS together (the coarse prefix) are accumulated directly: persistent
//     workgroups sweep the samples, merge runs of lanes that share a cell, add into an LDS copy of
//     those tables and flush it once;
//   * every other level is cut into bins of 8192 entries (128 KB of 64-bit sums in LDS).  A counting sweep
//     and a filling sweep over the samples (same persistent tiling, so each workgroup owns a private,
//     pre-computed slice of every bin's queue: no global atomics, no overflow) write one 16-byte record
//     (two entries within the bin, 4 values) per pair of corners along x, staged through LDS so that each
//     bin receives contiguous runs.  Then workgroups balanced by record count stream the queue,
//     accumulate in LDS (as scaled 64-bit integers: integer adds are the fastest LDS atomics) and add the
//     finished bin into dtable with coalesced atomics.
#include "encode_common.h"
#include <mutex>

namespace dg_encode_binned {

using namespace dg_encode;

constexpr int kChunkLog2 = 13;
constexpr uint32_t kChunk = 1u << kChunkLog2;      // entries per bin
constexpr int kMaxBins = 2048;                     // per level: 2^24 entries / 8192
constexpr int kTile = 512;                         // samples per tile == threads per binning workgroup
constexpr int kKeeper = 64;                        // narrow fill sweep: one more wavefront, which keeps the books of the 64 bins
constexpr int kPairs = kTile * 4;                  // records staged per (tile, level): one per pair of corners along x
constexpr uint32_t kMaxKeys = DG_MAX_LEVELS * kMaxBins;   // (level, bin) pairs at most: the count sweep keeps one counter each in LDS (128 KB)
constexpr int kBinGrid = 768;                      // persistent binning workgroups (three per compute unit)
constexpr int kAccBlock = 1024;                    // threads of an accumulate workgroup (one per compute unit: its table fills LDS)
constexpr int kAccDepth = 4;                       // records in flight per accumulate thread
constexpr int kAccRecordsLog2 = 17;
constexpr uint32_t kAccRecords = 1u << kAccRecordsLog2;   // an accumulate workgroup sums at least this many records of a bin (or all it has) ...
constexpr int kAccMaxLog2 = kAccRecordsLog2 + 1;          // ... and fewer than this many: a bin is cut into floor(records / kAccRecords) equal pieces
// pieces a bin of `total` records is cut into: a bin with less than two pieces' worth stays whole (a second workgroup
// would clear and write out a table of its own for little)
__host__ __device__ __forceinline__ uint32_t acc_pieces(uint32_t total) { return total == 0u ? 0u : (total >> kAccRecordsLog2 ? total >> kAccRecordsLog2 : 1u); }
constexpr int kCoarseBlock = 1024;                 // coarse prefix: threads per workgroup, persistent workgroups (one per compute unit)
constexpr int kCoarseGrid = 256;

struct Plan {
    uint32_t first_level;                  // levels below are accumulated directly in LDS
    uint32_t n_keys;                       // (level, bin) pairs of the binned levels
    uint32_t key_base[DG_MAX_LEVELS + 1];  // first key of each level
    uint32_t n_bins[DG_MAX_LEVELS];
    uint32_t max_bins;
};

// ------------------------------------------------------------------ coarse prefix: accumulate in LDS
__global__ void __launch_bounds__(kCoarseBlock)
coarse_kernel(dg_grid_desc g, uint32_t first_level, const float *__restrict__ u, const float2 *__restrict__ dfeat,
              uint64_t N, float *__restrict__ dtable)
{
    // 2 sums per entry of levels [0, first_level), one plane per feature (an add instruction then spreads over all LDS
    // banks); fp64 LDS atomics run ~7x faster than fp32 ones
    extern __shared__ double tab[];
    const uint32_t n_entries = g.offset[first_level], n_floats = 2u * n_entries;
    for (uint32_t i = threadIdx.x; i < n_floats; i += kCoarseBlock) tab[i] = 0.0;
    __syncthreads();
    const int lane = threadIdx.x % dg::kWave;
    const uint32_t mask = (1u << g.log2_T) - 1u;
    const uint64_t n_tiles = (N + kCoarseBlock - 1) / kCoarseBlock;
    for (uint64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const uint64_t n = tile * kCoarseBlock + threadIdx.x;
        const bool live = n < N;
        const uint64_t nn = live ? n : N - 1;
        const float uu[3] = {u[3 * nn], u[3 * nn + 1], u[3 * nn + 2]};
        for (uint32_t l = 0; l < first_level; ++l) {
            const LevelGeom lv = level_of(g, l);
            uint32_t cell[3], e[8];
            float frac[3], w[8];
            locate(lv, uu, cell, frac);
            corner_entries(lv, mask, cell, e);
            corner_weights(frac, w);
            float2 gfe = dfeat[(size_t)l * N + nn];
            if (!live) gfe = make_float2(0.0f, 0.0f);
            bool head = lane == 0;
#pragma unroll
            for (int a = 0; a < 3; ++a) head |= from_lane_below(cell[a]) != cell[a];
            const unsigned long long heads = __ballot(head);
            float vx[8], vy[8];
#pragma unroll
            for (int c = 0; c < 8; ++c) { vx[c] = w[c] * gfe.x; vy[c] = w[c] * gfe.y; }
            if (__popcll(heads) < dg::kWave) segmented_sum(vx, vy, head, heads);     // merge each run into its last lane
            const bool tail = lane == dg::kWave - 1 || ((heads >> ((lane + 1) & 63)) & 1ull);
            if (tail) {
#pragma unroll
                for (int c = 0; c < 8; ++c) {
                    const uint32_t slot = lv.offset + e[c];
                    if (vx[c] != 0.0f) __hip_atomic_fetch_add(&tab[slot], (double)vx[c], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    if (vy[c] != 0.0f) __hip_atomic_fetch_add(&tab[n_entries + slot], (double)vy[c], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                }
            }
        }
    }
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < n_floats; i += kCoarseBlock) {
        const float v = (float)tab[(i & 1u) * n_entries + (i >> 1)];
        if (v != 0.0f) unsafeAtomicAdd(dtable + i, v);
    }
}

// ------------------------------------------------------------------ binning sweeps
// One record serves a pair of corners along x: (entry of corner 0 within the bin, entry of corner 1
// within the bin, 4 values).  The two entries of a pair are neighbours in a dense level and differ only
// in their low index bits in a hashed one, so they share a bin -- except where the pair straddles a bin
// boundary (one pair in 8192 of a dense level).  Then the record carries corner 0 alone and corner 1 is
// added to the table directly with global atomics; both sweeps see exactly four records per emitting
// sample and level.

// A queue record is 16 bytes: the entry of corner 0 within the bin (13 bits), how corner 1's entry differs from it (4
// bits: the two differ in their k low bits, all of them -- x and x + 1 do, and both index forms keep that: a sum of
// x with multiples of the resolution, or an exclusive-or of x with hashes of y and z) and the pair's four values as
// 27-bit floats (sign, 8 exponent bits, 18 mantissa bits: fp32 rounded to nearest at bit 5, relative error at most
// 2^-20 per value, the same for both signs).  Sixteen bytes because eight of them make one 128-byte cache line: the narrow fill
// sweep appends in multiples of 8 records, so every append starts on a line boundary and covers whole lines; what
// does not fill a granule yet waits in LDS.  (With 20-byte records of fp32 values, probes of the store side alone
// measured 3.0 ms for 9.1 GB appended as it comes and 1.8 ms in whole lines; the fifth word, kept in a stream of its
// own, cost 2.5 times its share because its appends were fractions of a line.)
constexpr uint32_t kGran = 8;                         // append granule of the narrow fill sweep, in records
constexpr uint32_t kSliceRound = kGran;               // a workgroup's slice of a bin is padded to this many records (zero records)

// k such that eb == ea ^ (2^k - 1), or 15 when the two do not differ that way (ea, eb < 2^13)
__device__ __forceinline__ uint32_t pair_code(uint32_t ea, uint32_t eb)
{
    const uint32_t x = ea ^ eb, k = 32u - (uint32_t)__clz((int)x);       // __clz(0) == 32
    return x == (1u << k) - 1u ? k : 15u;
}

// (entry of corner 0 < 2^13, pair_code < 15, four values) <-> record.  A value keeps its top 27 bits, rounded to nearest
// (half a unit is added to the magnitude before the cut: ties go away from zero, the same way for both signs).
// x: entry, code and the low 15 bits of value 3; y, z, w: values 0..2 in the low 27 bits, more bits of value 3 above.
__device__ __forceinline__ uint4 pack_record(uint32_t ea, uint32_t code, float v0, float v1, float v2, float v3)
{
    const uint32_t q0 = (__float_as_uint(v0) + 16u) >> 5, q1 = (__float_as_uint(v1) + 16u) >> 5, q2 = (__float_as_uint(v2) + 16u) >> 5,
                   q3 = (__float_as_uint(v3) + 16u) >> 5;
    return make_uint4(ea | code << 13 | q3 << 17, q0 | (q3 >> 15) << 27, q1 | (q3 >> 20) << 27, q2 | (q3 >> 25) << 27);
}
template <typename R>
__device__ __forceinline__ void unpack_record(const R &r, uint32_t &ea, uint32_t &eb, float &v0, float &v1, float &v2, float &v3)
{
    ea = r.x & (kChunk - 1u);
    eb = ea ^ ((1u << (r.x >> 13 & 15u)) - 1u);
    v0 = __uint_as_float(r.y << 5);
    v1 = __uint_as_float(r.z << 5);
    v2 = __uint_as_float(r.w << 5);
    v3 = __uint_as_float((r.x >> 17 | (r.y >> 27) << 15 | (r.z >> 27) << 20 | (r.w >> 27) << 25) << 5);
}
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Which records a sample emits at a level (both sweeps take the same decision from the same data).  A
// wavefront holds 64 consecutive samples of a ray; lanes that share a cell form a run whose 16 values are
// summed into the run's last lane, which alone emits records.  Skipped where no two lanes share a cell.
struct Emission {
    uint32_t e[8];
    float frac[3];
    unsigned long long heads;
    bool head, merge, emit;
};

__device__ __forceinline__ Emission classify(const LevelGeom &lv, uint32_t mask, const float (&uu)[3], bool live, int lane)
{
    Emission o;
    uint32_t cell[3];
    locate(lv, uu, cell, o.frac);
    corner_entries(lv, mask, cell, o.e);
    o.head = lane == 0 || !live;
#pragma unroll
    for (int a = 0; a < 3; ++a) o.head |= from_lane_below(cell[a]) != cell[a];
    o.heads = __ballot(o.head);
    o.merge = __popcll(o.heads) < dg::kWave;      // any run at all: the merge steps cost less than the records they save
    const bool tail = lane == dg::kWave - 1 || ((o.heads >> ((lane + 1) & 63)) & 1ull);
    o.emit = live && (!o.merge || tail);
    return o;
}

// count sweep with this workgroup's counters in LDS: one LDS add per record, no barriers inside the sweep.  Launched
// with the fill sweep's grid and tiling: kTile threads that take one tile per step, or 2 * kTile that take two.
__global__ void __launch_bounds__(2 * kTile)
count_lds_kernel(dg_grid_desc g, Plan plan, const float *__restrict__ u, uint64_t n0, uint64_t nb, uint32_t *__restrict__ rows)
{
    extern __shared__ uint32_t smem[];
    uint32_t *row = smem;                                // [n_keys]
    const uint32_t tid = threadIdx.x, in_tile = tid % kTile;
    const int lane = tid % dg::kWave;
    const uint32_t mask = (1u << g.log2_T) - 1u;
    for (uint32_t i = tid; i < plan.n_keys; i += blockDim.x) row[i] = 0u;
    __syncthreads();
    const uint64_t n_tiles = (nb + kTile - 1) / kTile;
    const uint64_t stride = (uint64_t)(blockDim.x / kTile) * gridDim.x;
    for (uint64_t tile = blockIdx.x + (uint64_t)(tid / kTile) * gridDim.x; tile < n_tiles; tile += stride) {
        const uint64_t rel = tile * kTile + in_tile;
        const bool live = rel < nb;
        const uint64_t n = n0 + (live ? rel : nb - 1);
        const float uu[3] = {u[3 * n], u[3 * n + 1], u[3 * n + 2]};
        for (uint32_t l = plan.first_level; l < g.n_levels; ++l) {
            const Emission em = classify(level_of(g, l), mask, uu, live, lane);
            if (em.emit) {
                uint32_t *c = row + plan.key_base[l];
#pragma unroll
                for (int p = 0; p < 4; ++p) atomicAdd(&c[em.e[2 * p] >> kChunkLog2], 1u);
            }
        }
    }
    __syncthreads();
    uint32_t *row_global = rows + (size_t)blockIdx.x * plan.n_keys;
    for (uint32_t i = tid; i < plan.n_keys; i += blockDim.x) row_global[i] = row[i];
}

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ void scan_step(uint32_t &v)
{
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xF, true);
}

// inclusive prefix sum over the wavefront (DPP moves: rows of 16 lanes, then across rows)
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v)
{
    scan_step<0x111, 0xF>(v);
    scan_step<0x112, 0xF>(v);
    scan_step<0x114, 0xF>(v);
    scan_step<0x118, 0xF>(v);
    scan_step<0x142, 0xA>(v);
    scan_step<0x143, 0xC>(v);
    return v;
}

// inclusive running maximum over the wavefront, same moves (a lane that receives nothing takes 0)
__device__ __forceinline__ uint32_t wave_inclusive_max(uint32_t v)
{
#define DG_MAX_STEP(CTRL, ROW_MASK) v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xF, true))
    DG_MAX_STEP(0x111, 0xF); DG_MAX_STEP(0x112, 0xF); DG_MAX_STEP(0x114, 0xF); DG_MAX_STEP(0x118, 0xF);
    DG_MAX_STEP(0x142, 0xA); DG_MAX_STEP(0x143, 0xC);
#undef DG_MAX_STEP
    return v;
}

// Fill sweep.  Per step (one tile at one level): every emitting lane takes a rank in its records' bins (LDS
// counters), the counters are scanned into staging offsets, the records are staged in LDS sorted by bin and then
// copied to the queues, so that every bin receives contiguous runs.  A workgroup goes level after level, and
// within a level tile after tile: it then appends to the same queue slices step after step, so the partly written
// cache lines at their ends are completed while they still sit in L2.
// Loads are requested one step ahead: memory operations of a wavefront retire in order, so a load issued right
// after queue stores could only be awaited together with their acknowledgements.

struct StepAhead {
    float u[3];
    float2 g;
};

__device__ __forceinline__ void load_ahead(StepAhead &a, const float *__restrict__ u, const float2 *__restrict__ dfeat, uint64_t N,
                                           uint64_t n0, uint64_t nb, uint64_t tile, uint32_t l, uint32_t tid)
{
    const uint64_t rel = tile * kTile + tid, n = n0 + (rel < nb ? rel : nb - 1);
    a.u[0] = u[3 * n]; a.u[1] = u[3 * n + 1]; a.u[2] = u[3 * n + 2];
    a.g = dfeat[(size_t)l * N + n];
}

// values of the 8 corners of one sample at one level, runs merged where the emission says so; `largest` follows the
// largest magnitude (as the bit pattern of |v|, which orders like the value) of anything a lane emits
__device__ __forceinline__ void corner_values(const Emission &em, float2 gfe, float (&vx)[8], float (&vy)[8], uint32_t &largest)
{
    float w[8];
    corner_weights(em.frac, w);
#pragma unroll
    for (int c = 0; c < 8; ++c) { vx[c] = w[c] * gfe.x; vy[c] = w[c] * gfe.y; }
    if (em.merge) segmented_sum(vx, vy, em.head, em.heads);
    if (em.emit) {
        float m = 0.0f;
#pragma unroll
        for (int c = 0; c < 8; ++c) m = fmaxf(m, fmaxf(fabsf(vx[c]), fabsf(vy[c])));
        largest = max(largest, __float_as_uint(m));
    }
    // fmaxf passes over NaN: a NaN gradient is reported as such (its bit pattern orders above infinity's), by whichever
    // lane holds it, whether or not that lane emits
    if (gfe.x != gfe.x || gfe.y != gfe.y) largest = max(largest, 0x7fc00000u);
}

// largest over the workgroup -> *dst (one atomic per workgroup); `word` is an LDS word nobody else uses any more
__device__ __forceinline__ void publish_largest(uint32_t largest, uint32_t *word, uint32_t *__restrict__ dst)
{
    __syncthreads();
    if (threadIdx.x == 0) *word = 0u;
    __syncthreads();
#pragma unroll
    for (int off = dg::kWave / 2; off > 0; off >>= 1) largest = max(largest, (uint32_t)__shfl_xor((int)largest, off, dg::kWave));
    if (threadIdx.x % dg::kWave == 0 && largest) atomicMax(word, largest);
    __syncthreads();
    if (threadIdx.x == 0 && *word) atomicMax(dst, *word);
}

// the record of pair p; a pair that straddles a bin boundary (or, against every expectation, differs in some other way
// than a record can say) keeps corner 0 only and its corner 1 goes to the table directly
__device__ __forceinline__ uint4 make_record(const Emission &em, int p, const float (&vx)[8], const float (&vy)[8], uint32_t level_offset,
                                             float *__restrict__ dtable)
{
    const uint32_t ea = em.e[2 * p], eb = em.e[2 * p + 1];
    uint32_t code = pair_code(ea & (kChunk - 1u), eb & (kChunk - 1u));
    const bool together = (ea >> kChunkLog2) == (eb >> kChunkLog2) && code != 15u;
    if (!together) {
        code = 0u;
        float *dst = dtable + 2 * ((size_t)level_offset + eb);
        if (vx[2 * p + 1] != 0.0f) unsafeAtomicAdd(dst, vx[2 * p + 1]);
        if (vy[2 * p + 1] != 0.0f) unsafeAtomicAdd(dst + 1, vy[2 * p + 1]);
    }
    return pack_record(ea & (kChunk - 1u), code, vx[2 * p], vy[2 * p], together ? vx[2 * p + 1] : 0.0f, together ? vy[2 * p + 1] : 0.0f);
}

// Fill sweep for grids with at most 64 bins in every level.  kTile threads bin the samples; every one of their
// wavefronts reads the 64 step counters and scans them itself, so the staging offsets sit in one register per lane
// (lane == bin) and are fetched with wavefront shuffles.  The counters are double-buffered so that the buffer of the
// next step is cleared while this step is staged.  One more wavefront keeps the books (lane == bin): the queue
// position of every bin and the records that do not fill an append granule yet (up to 7 per bin, kept in LDS behind
// the staged ones, in two halves: one is read while the other is rebuilt).  While the others stage a step, it works
// out from the step's counters what every bin appends (whole granules) and publishes that; after the second barrier
// the binning threads copy the appends out, consecutive threads writing consecutive records of a bin, so that a store
// instruction covers whole cache lines, while the book-keeping wavefront puts together what waits from here on.  Two
// barriers per step.  At the end of a level the book-keeper writes the waiting records out and pads this workgroup's
// slice of each bin to kSliceRound records with zero records, which add nothing.
__device__ __forceinline__ uint32_t lane_value(uint32_t v, uint32_t lane) { return (uint32_t)__builtin_amdgcn_readlane((int)v, (int)lane); }

constexpr uint32_t kCarry = kGran - 1;
// append granules a step can hold: its records plus what waits in the 64 bins
constexpr uint32_t kOwner = ((kPairs + 64 * kCarry) / kGran + 1 + 3) / 4 * 4;
constexpr int kNarrowThreads = kTile + kKeeper;
constexpr int kNarrowLds = 128 * 4 + (kPairs + 2 * 64 * (int)kCarry) * 16 + 64 * 8 + 16 + (int)kOwner;

// K outputs per thread, all reads of a stage issued before the first is used.  Output f of the step belongs to the bin
// owner[f / kGran]; it is record j = f - before of the bin's append: one that waited while j < waiting, else a staged
// one (the waiting records lie behind the staged ones, from index `waited0` on).  bin_info[bin] = (before | waiting << 12 | first
// staging slot of the bin's fresh records << 16, queue position of the append).  Threads past the end repeat the last
// output (same value to the same place): no branch.  `total` must be positive.
template <int K>
__device__ __forceinline__ void copy_outputs(uint32_t base, uint32_t total, uint32_t tid, const uint8_t *owner, const uint2 *bin_info,
                                             const uint4 *stage, uint32_t waited0, uint4 *__restrict__ queue)
{
    uint32_t f[K], o[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        f[k] = min(base + k * kTile + tid, total - 1u);
        o[k] = owner[f[k] / kGran];
    }
    uint2 info[K];
#pragma unroll
    for (int k = 0; k < K; ++k) info[k] = bin_info[o[k]];
    uint32_t src[K], dst[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const uint32_t j = f[k] - (info[k].x & 4095u), waiting = info[k].x >> 12 & 15u, slot0 = info[k].x >> 16;
        const uint32_t staged = slot0 + j - waiting, waited = waited0 + o[k] * kCarry + j;
        const uint32_t pick = 0u - (uint32_t)(j < waiting);           // all ones: take the waiting record
        src[k] = staged ^ ((staged ^ waited) & pick);
        dst[k] = info[k].y + j;
    }
    uint4 rec[K];
#pragma unroll
    for (int k = 0; k < K; ++k) rec[k] = stage[src[k]];
#pragma unroll
    for (int k = 0; k < K; ++k) queue[dst[k]] = rec[k];
}

// the step's appends -> queue, by the kTile binning threads (the trip counts are the same for all)
__device__ __forceinline__ void copy_step(uint32_t total, uint32_t tid, const uint8_t *owner, const uint2 *bin_info, const uint4 *stage,
                                          uint32_t waited0, uint4 *__restrict__ queue)
{
    for (uint32_t base = 0; base < total;) {
        const uint32_t rounds = (total - base + kTile - 1) / kTile;
#define DG_COPY(K) copy_outputs<K>(base, total, tid, owner, bin_info, stage, waited0, queue)
        if (rounds >= 4) { DG_COPY(4); base += 4 * kTile; }
        else if (rounds == 3) { DG_COPY(3); break; }
        else if (rounds == 2) { DG_COPY(2); break; }
        else { DG_COPY(1); break; }
#undef DG_COPY
    }
}

__global__ void __launch_bounds__(kNarrowThreads, 7)     // three workgroups of nine wavefronts per compute unit: seven wavefronts per SIMD
fill_narrow_kernel(dg_grid_desc g, Plan plan, const float *__restrict__ u, const float2 *__restrict__ dfeat, uint64_t N,
                   uint64_t n0, uint64_t nb, const uint32_t *__restrict__ rows, const uint32_t *__restrict__ binbase,
                   uint4 *__restrict__ queue, float *__restrict__ dtable, uint32_t *__restrict__ largest_out)
{
    extern __shared__ uint32_t smem[];
    uint32_t *cnt = smem;                                             // [2][64] records per bin of the step
    uint4 *stage = reinterpret_cast<uint4 *>(cnt + 128);              // [kPairs] records of the step, sorted by bin
    uint4 *carry = stage + kPairs;                                    // [2][64][kCarry] what waits, per bin: read in one half, rebuilt in the other
    uint2 *bin_info = reinterpret_cast<uint2 *>(carry + 2 * 64 * kCarry);          // [64] see copy_outputs
    uint32_t *total_out = reinterpret_cast<uint32_t *>(bin_info + 64);             // [1] outputs of the step (+ 3 unused)
    uint8_t *owner = reinterpret_cast<uint8_t *>(total_out + 4);      // [kOwner] bin of each granule of the step
    const uint32_t tid = threadIdx.x;
    const bool keeper = tid >= (uint32_t)kTile;                       // the last wavefront: kTile is a multiple of 64
    const uint32_t lane = tid % dg::kWave;
    const uint32_t mask = (1u << g.log2_T) - 1u;
    const uint32_t *row_global = rows + (size_t)blockIdx.x * plan.n_keys;
    if (tid < 128) cnt[tid] = 0u;
    __syncthreads();
    uint32_t parity = 0, largest = 0;
    const uint64_t n_tiles = (nb + kTile - 1) / kTile;
    const bool has_work = blockIdx.x < n_tiles;

    if (keeper) {
        // lane b keeps the books of bin b: where its next append goes and how many records wait
        uint32_t pos = 0, waiting = 0;
        const uint4 zero4 = make_uint4(0u, 0u, 0u, 0u);
        for (uint32_t l = plan.first_level; l < g.n_levels; ++l) {
            const uint32_t n_bins = plan.n_bins[l], key0 = plan.key_base[l];
            const bool mine = lane < n_bins;
            if (mine) pos = binbase[key0 + lane] + row_global[key0 + lane];
            for (uint64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x, parity ^= 1u) {
                __syncthreads();                                     // ranks taken
                // from what waits and what is fresh: how much goes out (whole granules) and how much is left; the
                // granules of all bins laid end to end, with a table of which bin owns each
                const uint32_t fresh = cnt[64u * parity + lane];
                const uint32_t slot0 = wave_inclusive_scan(fresh) - fresh;
                const uint32_t have = waiting + fresh, out = have & ~(kGran - 1u), left = have - out;
                const uint32_t incl = wave_inclusive_scan(out), before = incl - out;
                const uint32_t total = lane_value(incl, dg::kWave - 1);
                if (n_bins > 16) {
                    for (uint32_t q = 0; q < out / kGran; ++q) owner[before / kGran + q] = (uint8_t)lane;
                } else {
                    // few bins, long appends: every bin marks its first granule, a running maximum spreads the marks
                    // (bins come in rising order; bin 0 is what an unmarked granule reads)
                    const uint32_t n_gran = total / kGran;
                    for (uint32_t g0 = 0; g0 < n_gran; g0 += dg::kWave)
                        if (g0 + lane < n_gran) owner[g0 + lane] = 0;
                    if (out) owner[before / kGran] = (uint8_t)lane;
                    uint32_t run = 0;
                    for (uint32_t g0 = 0; g0 < n_gran; g0 += dg::kWave) {
                        const uint32_t v = max(run, wave_inclusive_max(g0 + lane < n_gran ? owner[g0 + lane] : 0u));
                        if (g0 + lane < n_gran) owner[g0 + lane] = (uint8_t)v;
                        run = lane_value(v, dg::kWave - 1);
                    }
                }
                bin_info[lane] = make_uint2(before | waiting << 12 | slot0 << 16, pos);
                if (lane == 0) *total_out = total;
                __syncthreads();                                     // step staged, plan published
                // While the others copy the appends out, the records that wait from here on are put together in the
                // other half of the waiting slots.  Nothing went out (out == 0): those that waited stay, the fresh ones
                // queue up behind them; else all that waited leaves and the tail of the fresh ones waits.  A value
                // beyond what waits is written back to where it was read: straight-line code, no branch per record;
                // all reads first, then all writes (named values: an array of 16-byte values ends up in scratch
                // memory here).
                {
                    const uint32_t keep = out == 0u ? waiting : 0u, fresh_from = out == 0u ? slot0 : slot0 + (out - waiting);
                    const uint32_t old_at = kPairs + parity * 64u * kCarry + lane * kCarry, new_at = kPairs + (parity ^ 1u) * 64u * kCarry + lane * kCarry;
                    static_assert(kCarry == 7, "the moves below are written out for seven waiting records");
#define DG_FROM(j) (j##u < keep ? old_at + j##u : min(fresh_from + (j##u - keep), (uint32_t)kPairs - 1u))
                    const uint4 r0 = stage[DG_FROM(0)], r1 = stage[DG_FROM(1)], r2 = stage[DG_FROM(2)], r3 = stage[DG_FROM(3)];
                    const uint4 r4 = stage[DG_FROM(4)], r5 = stage[DG_FROM(5)], r6 = stage[DG_FROM(6)];
#define DG_MOVE(j) stage[j##u < left ? new_at + j##u : DG_FROM(j)] = r##j
                    DG_MOVE(0); DG_MOVE(1); DG_MOVE(2); DG_MOVE(3); DG_MOVE(4); DG_MOVE(5); DG_MOVE(6);
#undef DG_MOVE
#undef DG_FROM
                    pos += out;
                    waiting = left;
                }
            }
            // end of the level: what still waits goes out, followed by zero records up to the padded end of the slice
            if (mine) {
                const uint32_t end = (pos + waiting + kSliceRound - 1u) / kSliceRound * kSliceRound;
                for (uint32_t j = 0; pos + j < end; ++j) queue[pos + j] = j < waiting ? carry[(parity * 64u + lane) * kCarry + j] : zero4;
            }
            waiting = 0u;
        }
        publish_largest(0u, cnt, largest_out);
        return;
    }

    StepAhead ahead = {{0.0f, 0.0f, 0.0f}, make_float2(0.0f, 0.0f)};
    if (has_work) load_ahead(ahead, u, dfeat, N, n0, nb, blockIdx.x, plan.first_level, tid);
    // taken in before the loop, as every later load is before its step ends: the top of a step then waits for nothing
    asm volatile("" : "+v"(ahead.u[0]), "+v"(ahead.u[1]), "+v"(ahead.u[2]), "+v"(ahead.g.x), "+v"(ahead.g.y));
    for (uint32_t l = plan.first_level; l < g.n_levels; ++l) {
        const LevelGeom lv = level_of(g, l);
        for (uint64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x, parity ^= 1u) {
            uint32_t *c_cur = cnt + 64u * parity;
            const bool live = tile * kTile + tid < nb;
            const float uu[3] = {ahead.u[0], ahead.u[1], ahead.u[2]};
            const float2 gfe = live ? ahead.g : make_float2(0.0f, 0.0f);
            // The next step's inputs are asked for right away and taken in at the end of the staging: the whole step
            // hides their latency.  (Asked for after the copy, the wait for them would also wait for the copy's
            // stores, which have only just been issued.)
            {
                const bool same_level = tile + gridDim.x < n_tiles;
                const uint32_t l_next = same_level ? l : l + 1;
                if (l_next < g.n_levels) load_ahead(ahead, u, dfeat, N, n0, nb, same_level ? tile + gridDim.x : blockIdx.x, l_next, tid);
            }
            const Emission em = classify(lv, mask, uu, live, (int)lane);
            uint32_t rank[4];
            if (em.emit) {
#pragma unroll
                for (int p = 0; p < 4; ++p) rank[p] = atomicAdd(&c_cur[em.e[2 * p] >> kChunkLog2], 1u);
            }
            float vx[8], vy[8];
            corner_values(em, gfe, vx, vy, largest);                     // needs no rank: done while the books of the last step are closed
            __syncthreads();
            // lane b: records of bin b in this step and their first staging slot
            const uint32_t in_bin = c_cur[lane];
            const uint32_t first_slot = wave_inclusive_scan(in_bin) - in_bin;
            if (tid < dg::kWave) cnt[64u * (parity ^ 1u) + tid] = 0u;    // the other buffer: last read two barriers ago
            uint32_t slot[4];
#pragma unroll
            for (int p = 0; p < 4; ++p) slot[p] = __shfl(first_slot, (int)(em.e[2 * p] >> kChunkLog2), dg::kWave);
            if (em.emit) {
#pragma unroll
                for (int p = 0; p < 4; ++p) stage[slot[p] + rank[p]] = make_record(em, p, vx, vy, lv.offset, dtable);
            }
            // the inputs are taken in here, before this wavefront issues stores again (an empty statement that uses them)
            asm volatile("" : "+v"(ahead.u[0]), "+v"(ahead.u[1]), "+v"(ahead.u[2]), "+v"(ahead.g.x), "+v"(ahead.g.y));
            __syncthreads();
            copy_step(*total_out, tid, owner, bin_info, stage, kPairs + parity * 64u * kCarry, queue);
        }
    }
    publish_largest(largest, cnt, largest_out);
}

// Fill sweep for many bins, appends in 64-byte granules.  Memory takes a lone 16-byte record badly (measured on this
// chip with 2048 open queue slices per workgroup: 72 G records/s as single records, 208 G/s as aligned groups of four
// written by four neighbouring lanes, 295 G/s as whole lines), and with thousands of bins a step brings a bin one
// record or none, so the groups have to be collected over several steps.  One workgroup of 1024 threads per compute
// unit keeps, for every bin of the level, the granule its queue slice is being filled at: four record slots in LDS
// (128 KB for 2048 bins), the position of the bin's next record, and the position `from` which the granule is kept
// in LDS (records of the granule below that were written to memory directly).
// A step bins two tiles of 512 samples, in rounds of one pair of corners each.  Phase 1 of a round: every record takes
// its queue position with an LDS add on the bin's counter (the count sweep has sized this workgroup's slice of every
// bin for exactly its records, and integer sums do not care in which order lanes take positions); a position inside
// the bin's granule puts the record into its LDS slot, and the record that takes the granule's last position enters
// the bin into the round's list; a position beyond the granule (the bin got more in this round than its granule had
// room for) is written to the queue directly.  Phase 2, after a barrier: groups of four lanes write the listed
// granules out, one 64-byte store per group, and move the bin on to the granule of its counter -- what lies between
// was written directly.  A second barrier keeps the next round's records off the slots until they have been read.
// At the end of a level the granules that are still open go out, filled up with zero records, which add nothing; the
// count sweep has sized every slice in whole granules for that.  Levels with few bins see many records per bin and
// round, most of which go to the queue directly -- into few open cache lines, which L2 completes (226 G records/s
// measured for lone records into 64 slices per workgroup).
// Measured at T = 2^24 (19.8 M samples, 14 binned levels, 2048 bins in seven of them): records sorted per step in LDS
// and copied out 10.7 ms, every record stored directly 10.2 ms, granules with all four pairs in one round 8.0 ms, two
// rounds 7.4 ms, four rounds 7.1 ms.
constexpr int kRingThreads = 1024, kRingGrid = 256, kRingSlots = 4, kRingRounds = 4;
constexpr int kRingLds = kMaxBins * (kRingSlots * 16 + 4 + 4 + 2 * 2) + 16;

__global__ void __launch_bounds__(kRingThreads)
fill_ring_kernel(dg_grid_desc g, Plan plan, const float *__restrict__ u, const float2 *__restrict__ dfeat, uint64_t N,
                 uint64_t n0, uint64_t nb, const uint32_t *__restrict__ rows, const uint32_t *__restrict__ binbase,
                 uint4 *__restrict__ queue, float *__restrict__ dtable, uint32_t *__restrict__ largest_out)
{
    extern __shared__ uint32_t smem[];
    const uint32_t cap = plan.max_bins;
    uint4 *ring = reinterpret_cast<uint4 *>(smem);                    // [cap][4] the granule each bin is being filled at
    uint32_t *pos = smem + (size_t)cap * kRingSlots * 4;              // [cap] queue position of the bin's next record
    uint32_t *from = pos + cap;                                       // [cap] the granule is in LDS from this position on
    uint32_t *n_list = from + cap;                                    // [2] entries of the two lists (+ 2 unused words)
    uint16_t *list = reinterpret_cast<uint16_t *>(n_list + 4);        // [2][cap] bins whose granule filled up in a step
    const uint32_t tid = threadIdx.x;
    const int lane = tid % dg::kWave;
    const uint32_t half = tid / kTile, in_tile = tid % kTile;         // the workgroup takes two tiles per step
    const uint32_t mask = (1u << g.log2_T) - 1u;
    const uint32_t *row = rows + (size_t)blockIdx.x * plan.n_keys;
    const uint4 zero4 = make_uint4(0u, 0u, 0u, 0u);
    uint32_t largest = 0, parity = 0;
    const uint64_t n_tiles = (nb + kTile - 1) / kTile;
    const uint64_t stride = 2ull * gridDim.x;                         // tiles between two steps of one half
    const uint64_t first_tile = blockIdx.x + (uint64_t)half * gridDim.x;
    // steps of the workgroup: until its first half runs out of tiles (the second half's tiles come later in the order)
    const uint64_t n_steps = blockIdx.x < n_tiles ? (n_tiles - blockIdx.x + stride - 1) / stride : 0;
    StepAhead ahead = {{0.0f, 0.0f, 0.0f}, make_float2(0.0f, 0.0f)};
    if (first_tile < n_tiles) load_ahead(ahead, u, dfeat, N, n0, nb, first_tile, plan.first_level, in_tile);
    if (tid < 2) n_list[tid] = 0u;
    for (uint32_t l = plan.first_level; l < g.n_levels; ++l) {
        const uint32_t n_bins = plan.n_bins[l], key0 = plan.key_base[l];
        const LevelGeom lv = level_of(g, l);
        __syncthreads();                                              // the last level's books are closed
        for (uint32_t i = tid; i < n_bins; i += kRingThreads) { const uint32_t p0 = row[key0 + i] + binbase[key0 + i]; pos[i] = p0; from[i] = p0; }
        __syncthreads();
        for (uint64_t step = 0; step < n_steps; ++step) {
            const uint64_t tile = first_tile + step * stride;
            const bool in_range = tile < n_tiles;
            const bool live = in_range && tile * kTile + in_tile < nb;
            const float uu[3] = {ahead.u[0], ahead.u[1], ahead.u[2]};
            const float2 gfe = live ? ahead.g : make_float2(0.0f, 0.0f);
            // the next step's inputs are asked for before this step's stores (loads and stores of a wavefront retire in order)
            {
                const bool same_level = step + 1 < n_steps;
                const uint32_t l_next = same_level ? l : l + 1;
                const uint64_t t_next = same_level ? tile + stride : first_tile;
                if (l_next < g.n_levels && t_next < n_tiles) load_ahead(ahead, u, dfeat, N, n0, nb, t_next, l_next, in_tile);
            }
            const Emission em = classify(lv, mask, uu, live, lane);
            float vx[8], vy[8];
            corner_values(em, gfe, vx, vy, largest);
            // The step's records go in kRingRounds rounds, each followed by its own write-out: the fewer records a bin
            // gets per round, the less often its granule overflows and records go to the queue one by one.
#pragma unroll
            for (int round = 0; round < kRingRounds; ++round, parity ^= 1u) {
                constexpr int kPer = 4 / kRingRounds;                 // pairs of corners per round
                uint16_t *mine = list + parity * cap;
                uint32_t at[kPer], end[kPer];                         // position of each record, end of its bin's granule
                if (em.emit) {
#pragma unroll
                    for (int k = 0; k < kPer; ++k) {
                        const uint32_t bin = em.e[2 * (kPer * round + k)] >> kChunkLog2;
                        at[k] = atomicAdd(&pos[bin], 1u);
                        end[k] = (from[bin] & ~(kRingSlots - 1u)) + kRingSlots;
                    }
#pragma unroll
                    for (int k = 0; k < kPer; ++k) {
                        const uint32_t bin = em.e[2 * (kPer * round + k)] >> kChunkLog2;
                        const uint4 rec = make_record(em, kPer * round + k, vx, vy, lv.offset, dtable);
                        if (at[k] < end[k]) ring[bin * kRingSlots + (at[k] & (kRingSlots - 1u))] = rec;
                        else queue[at[k]] = rec;
                    }
                }
                // bins whose granule this round completes go into the list: one LDS add per wavefront and pair of corners,
                // not one per bin (hundreds of adds on one word would take turns)
#pragma unroll
                for (int k = 0; k < kPer; ++k) {
                    const bool full = em.emit && at[k] == end[k] - 1u;
                    const unsigned long long votes = __ballot(full);
                    if (votes) {                                      // wavefront-uniform
                        const int leader = __ffsll((long long)votes) - 1;
                        uint32_t first = 0;
                        if (lane == leader) first = atomicAdd(&n_list[parity], (uint32_t)__popcll(votes));
                        first = lane_value(first, (uint32_t)leader);
                        if (full) mine[first + __popcll(votes & ((1ull << lane) - 1ull))] = (uint16_t)(em.e[2 * (kPer * round + k)] >> kChunkLog2);
                    }
                }
                __syncthreads();                                      // slots written, list complete
                {
                    const uint32_t n = n_list[parity], slot = tid % kRingSlots;
                    for (uint32_t i = tid / kRingSlots; i < n; i += kRingThreads / kRingSlots) {
                        const uint32_t bin = mine[i];
                        const uint32_t kept = from[bin], first = kept & ~(kRingSlots - 1u);
                        const uint4 rec = ring[bin * kRingSlots + slot];
                        if (first + slot >= kept) queue[first + slot] = rec;
                        if (slot == 0) from[bin] = pos[bin];          // what lies between went to the queue directly
                    }
                    if (tid == 0) n_list[parity ^ 1u] = 0u;           // the other list: last read before the barrier above
                }
                __syncthreads();                                      // slots read, bins moved on
            }
        }
        // end of the level: open granules go out, filled up with zero records
        {
            const uint32_t slot = tid % kRingSlots;
            for (uint32_t bin = tid / kRingSlots; bin < n_bins; bin += kRingThreads / kRingSlots) {
                const uint32_t kept = from[bin], first = kept & ~(kRingSlots - 1u), next = pos[bin], at = first + slot;
                if (next > first && at >= kept) queue[at] = at < next ? ring[bin * kRingSlots + slot] : zero4;
            }
        }
    }
    publish_largest(largest, n_list, largest_out);
}

// rows[b][k] (per-workgroup counts, each rounded up to a multiple of `round`) -> exclusive prefix over workgroups;
// totals[k].  A workgroup serves 32 keys; 32 groups of threads each take a contiguous stretch of the rows.
constexpr int kScanKeys = 32, kScanGroups = 32;
__global__ void __launch_bounds__(kScanKeys * kScanGroups)
scan_rows_kernel(uint32_t *__restrict__ rows, uint32_t n_rows, uint32_t n_keys, uint32_t round, uint32_t *__restrict__ totals)
{
    __shared__ uint32_t part[kScanGroups][kScanKeys];
    const uint32_t col = threadIdx.x % kScanKeys, group = threadIdx.x / kScanKeys;
    const uint32_t k = blockIdx.x * kScanKeys + col;
    const uint32_t per = (n_rows + kScanGroups - 1) / kScanGroups;
    const uint32_t lo = min(group * per, n_rows), hi = min(lo + per, n_rows);
    uint32_t sum = 0;
    if (k < n_keys)
        for (uint32_t b = lo; b < hi; ++b) sum += (rows[(size_t)b * n_keys + k] + round - 1u) / round * round;
    part[group][col] = sum;
    __syncthreads();
    if (k >= n_keys) return;
    uint32_t run = 0;
    for (uint32_t g = 0; g < group; ++g) run += part[g][col];
    for (uint32_t b = lo; b < hi; ++b) {
        const uint32_t t = (rows[(size_t)b * n_keys + k] + round - 1u) / round * round;     // a slice is padded to whole granules
        rows[(size_t)b * n_keys + k] = run;
        run += t;
    }
    if (group == kScanGroups - 1) totals[k] = run;
}

// binbase = exclusive scan of totals; blkbase = exclusive scan of the number of accumulate workgroups each
// bin gets (acc_pieces of its record count), so that work is balanced whatever the bins hold
// (one workgroup; n_keys is at most a few tens of thousands)
__global__ void __launch_bounds__(1024)
scan_totals_kernel(const uint32_t *__restrict__ totals, uint32_t n_keys, uint32_t *__restrict__ binbase,
                   uint32_t *__restrict__ blkbase)
{
    __shared__ uint32_t part[1024], part_b[1024];
    const uint32_t per = (n_keys + 1023) / 1024, lo = threadIdx.x * per;
    uint32_t s = 0, sb = 0;
    for (uint32_t i = lo; i < lo + per && i < n_keys; ++i) { s += totals[i]; sb += acc_pieces(totals[i]); }
    part[threadIdx.x] = s;
    part_b[threadIdx.x] = sb;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t run = 0, run_b = 0;
        for (int i = 0; i < 1024; ++i) {
            const uint32_t t = part[i], tb = part_b[i];
            part[i] = run; part_b[i] = run_b;
            run += t; run_b += tb;
        }
        binbase[n_keys] = run;
        binbase[n_keys + 1] = 0u;        // the fill sweep leaves the largest record magnitude of the batch here
        blkbase[n_keys] = run_b;
    }
    __syncthreads();
    uint32_t run = part[threadIdx.x], run_b = part_b[threadIdx.x];
    for (uint32_t i = lo; i < lo + per && i < n_keys; ++i) {
        binbase[i] = run; blkbase[i] = run_b;
        run += totals[i]; run_b += acc_pieces(totals[i]);
    }
}

// ------------------------------------------------------------------ accumulate one (bin, split)
// The sums are kept as 64-bit integers in LDS: integer adds there run at almost twice the rate of fp64 adds
// (2.7 against 1.5 T adds/s measured).  A value v becomes round(v * 2^k) with k chosen from the largest record
// magnitude of the batch so that the sum of a workgroup's records (fewer than 2^kAccMaxLog2) stays below 2^50; the
// conversion is the add of 1.5 * 2^52 in fp64, after which the low mantissa bits hold the integer in two's complement.
// The quantum is 2^-31 of the largest magnitude or finer, hundreds of times below the fp32 rounding of the value itself,
// and integer sums do not depend on the order of the additions.
constexpr double kIntegerMagic = 6755399441055744.0;     // 1.5 * 2^52

__device__ __forceinline__ void add_fixed(unsigned long long *slot, float v, double scale)
{
    const double shifted = __builtin_fma((double)v, scale, kIntegerMagic);
    const long long q = (long long)__double_as_longlong(shifted) - (long long)__double_as_longlong(kIntegerMagic);
    __hip_atomic_fetch_add(slot, (unsigned long long)q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

__global__ void __launch_bounds__(kAccBlock)
accumulate_kernel(dg_grid_desc g, Plan plan, const uint32_t *__restrict__ binbase, const uint32_t *__restrict__ blkbase,
                  const u32x4 *__restrict__ queue, float *__restrict__ dtable)
{
    // [2][kChunk] sums, one plane per feature: an add instruction then spreads over all LDS banks instead of every other pair
    extern __shared__ unsigned long long acc_tab[];
    unsigned long long *tab = acc_tab;
    if (blockIdx.x >= blkbase[plan.n_keys]) return;
    // the bin this workgroup serves: last key whose first workgroup is <= blockIdx.x
    uint32_t lo_k = 0, hi_k = plan.n_keys;
    while (hi_k - lo_k > 1) {
        const uint32_t mid = (lo_k + hi_k) / 2;
        if (blkbase[mid] <= blockIdx.x) lo_k = mid; else hi_k = mid;
    }
    const uint32_t key = lo_k, part = blockIdx.x - blkbase[key];
    // this workgroup's piece of the bin: the bin's records in equal shares (fewer than 2^kAccMaxLog2 each)
    const uint32_t total = binbase[key + 1] - binbase[key], pieces = blkbase[key + 1] - blkbase[key];
    const uint32_t share = (total + pieces - 1u) / pieces;
    const size_t begin = (size_t)binbase[key] + (size_t)part * share;
    const size_t end = min(begin + (size_t)share, (size_t)binbase[key + 1]);
    // 2^k with k = 50 - kAccMaxLog2 - 1 - (exponent of the largest magnitude): 2^kAccMaxLog2 values of that size sum to < 2^50
    const uint32_t top = binbase[plan.n_keys + 1] >> 23;                 // biased exponent (0 for zero / denormal: no smaller k needed)
    const int k = 50 - kAccMaxLog2 - 1 - ((int)(top ? top : 1u) - 127);
    const double scale = __longlong_as_double((long long)(1023 + k) << 52);
    const double inv_scale = __longlong_as_double((long long)(1023 - k) << 52);
    if (top == 255u) {
        // an infinite or NaN contribution somewhere in the batch: the scale above means nothing and integer sums cannot
        // carry it.  The gradient is marked instead: every bin that has records gets NaN in its first entry, as sums
        // with fp32 atomics would end up non-finite too.
        if (threadIdx.x == 0 && begin < end) {
            uint32_t lv = plan.first_level;
            while (lv + 1 < g.n_levels && key >= plan.key_base[lv + 1]) ++lv;
            dtable[2 * ((size_t)g.offset[lv] + (size_t)(key - plan.key_base[lv]) * kChunk)] = __uint_as_float(0x7fc00000u);
        }
        return;
    }
    for (uint32_t i = threadIdx.x; i < 2 * kChunk; i += kAccBlock) tab[i] = 0ull;
    __syncthreads();
    // several records in flight per thread so that the queue streams at memory speed: the loads are unconditional
    // (index clamped into the range) so that they issue back to back; a clamped duplicate adds 0
    if (begin < end) {
        const size_t last = end - 1;
        for (size_t i0 = begin + threadIdx.x; i0 < end; i0 += kAccDepth * kAccBlock) {
            u32x4 rec[kAccDepth];
#pragma unroll
            for (int k2 = 0; k2 < kAccDepth; ++k2) {
                const size_t want = i0 + (size_t)k2 * kAccBlock, i = want < last ? want : last;
                rec[k2] = __builtin_nontemporal_load(queue + i);      // read once: streams faster past the caches (measured)
            }
#pragma unroll
            for (int k2 = 0; k2 < kAccDepth; ++k2) {
                if (!(i0 + (size_t)k2 * kAccBlock < end)) rec[k2] = u32x4{0u, 0u, 0u, 0u};      // a clamped duplicate: the zero record
                uint32_t ea, eb;
                float v0, v1, v2, v3;
                unpack_record(rec[k2], ea, eb, v0, v1, v2, v3);
                add_fixed(&tab[ea], v0, scale);
                add_fixed(&tab[kChunk + ea], v1, scale);
                add_fixed(&tab[eb], v2, scale);
                add_fixed(&tab[kChunk + eb], v3, scale);
            }
        }
    }
    __syncthreads();
    uint32_t l = plan.first_level;
    while (l + 1 < g.n_levels && key >= plan.key_base[l + 1]) ++l;
    const uint32_t bin = key - plan.key_base[l];
    const uint32_t level_len = g.offset[l + 1] - g.offset[l];
    const uint32_t first = bin * kChunk, n_valid = min(kChunk, level_len - first);
    float *dst = dtable + 2 * ((size_t)g.offset[l] + first);
    for (uint32_t i = threadIdx.x; i < 2 * n_valid; i += kAccBlock) {
        const long long sum = (long long)tab[(i & 1u) * kChunk + (i >> 1)];
        if (sum != 0) {
            // |sum| < 2^50: high and low halves convert exactly
            const double wide = (double)(int)(sum >> 32) * 4294967296.0 + (double)(uint32_t)sum;
            unsafeAtomicAdd(dst + i, (float)(wide * inv_scale));
        }
    }
}

Plan make_plan(const dg_grid_desc *d)
{
    Plan p{};
    uint32_t l = 0;
    while (l < d->n_levels && d->offset[l + 1] <= kChunk) ++l;     // coarse prefix: tables that fit LDS together
    p.first_level = l;
    uint32_t key = 0;
    for (; l < d->n_levels; ++l) {
        p.key_base[l] = key;
        p.n_bins[l] = (d->offset[l + 1] - d->offset[l] + kChunk - 1) / kChunk;
        key += p.n_bins[l];
        if (p.n_bins[l] > p.max_bins) p.max_bins = p.n_bins[l];
    }
    p.max_bins = (p.max_bins + 63) / 64 * 64;
    p.key_base[d->n_levels] = key;
    p.n_keys = key;
    return p;
}

inline size_t align256(size_t x) { return (x + 255) / 256 * 256; }

struct Layout {
    size_t rows, totals, binbase, blkbase, queue, total;
    uint64_t batch;      // samples per batch
    uint64_t records;    // queue capacity: the records of a batch plus the padding of the slices
};

// both sweeps pad every workgroup's slice of every bin to whole granules: 8 records with few bins, 4 with many
uint32_t sweep_grid(const Plan &p) { return p.max_bins <= 64 ? (uint32_t)kBinGrid : (uint32_t)kRingGrid; }
uint32_t slice_round(const Plan &p) { return p.max_bins <= 64 ? kSliceRound : (uint32_t)kRingSlots; }
uint64_t slice_padding(const Plan &p) { return (uint64_t)sweep_grid(p) * p.n_keys * (slice_round(p) - 1u); }

// workspace layout for a batch of `batch` samples
Layout make_layout(const dg_grid_desc *d, const Plan &p, uint64_t batch)
{
    Layout L{};
    const uint64_t records = (batch * 4ull * (d->n_levels - p.first_level) + slice_padding(p) + 15ull) / 16ull * 16ull;
    size_t off = 0;
    L.rows = off; off = align256(off + (size_t)sweep_grid(p) * p.n_keys * 4);
    L.totals = off; off = align256(off + (size_t)p.n_keys * 4);
    L.binbase = off; off = align256(off + (size_t)(p.n_keys + 2) * 4);      // + the largest record magnitude
    L.blkbase = off; off = align256(off + (size_t)(p.n_keys + 1) * 4);
    L.queue = off; off = align256(off + records * 16);
    L.total = off;
    L.batch = batch;
    L.records = records;
    return L;
}

uint64_t max_batch(const dg_grid_desc *d, const Plan &p)
{
    const uint64_t per_sample = 4ull * (d->n_levels - p.first_level);
    if (per_sample == 0) return ~0ull;
    return ((0xffffffffull - slice_padding(p) - 16ull) / per_sample) / kTile * kTile;           // record offsets stay below 2^32
}

}  // namespace dg_encode_binned

namespace dg {

size_t encode_bwd_binned_workspace_bytes(const dg_grid_desc *d, uint64_t N)
{
    using namespace dg_encode_binned;
    const Plan p = make_plan(d);
    if (p.n_keys == 0) return 256;
    uint64_t batch = (N + kTile - 1) / kTile * kTile;
    const uint64_t cap = max_batch(d, p);
    if (batch > cap) batch = cap;
    if (batch == 0) batch = kTile;
    return make_layout(d, p, batch).total;
}

namespace {

using namespace dg_encode_binned;

// what a call works with: the plan of the grid, the batch the workspace holds and the workspace's parts
struct Prepared {
    Plan p;
    Layout L;
    uint32_t *rows, *totals, *binbase, *blkbase;
    uint4 *queue;
    uint32_t grid;
    bool narrow;
};

int prepare(const char *who, const dg_grid_desc *d, uint64_t N, void *ws, size_t ws_bytes, Prepared &q)
{
    q.p = make_plan(d);
    // kernels that use more LDS than a launch gets by default: asked for once per process, whichever thread comes first
    static std::once_flag lds_once;
    static hipError_t lds_status = hipSuccess;
    std::call_once(lds_once, [] {
        const int acc_lds = 2 * kChunk * (int)sizeof(double), count_lds = (int)kMaxKeys * 4;
        const hipError_t e[5] = {
            hipFuncSetAttribute(reinterpret_cast<const void *>(&fill_ring_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, kRingLds),
            hipFuncSetAttribute(reinterpret_cast<const void *>(&count_lds_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, count_lds),
            hipFuncSetAttribute(reinterpret_cast<const void *>(&fill_narrow_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, kNarrowLds),
            hipFuncSetAttribute(reinterpret_cast<const void *>(&accumulate_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, acc_lds),
            hipFuncSetAttribute(reinterpret_cast<const void *>(&coarse_kernel), hipFuncAttributeMaxDynamicSharedMemorySize, acc_lds)};
        for (const hipError_t x : e)
            if (x != hipSuccess) lds_status = x;
    });
    if (lds_status != hipSuccess) return dg::fail(DG_ERR_HIP, "%s: cannot reserve LDS: %s", who, hipGetErrorString(lds_status));
    if (q.p.n_keys == 0) return DG_OK;
    if (q.p.n_keys > kMaxKeys) return dg::fail(DG_ERR_UNSUPPORTED, "%s: %u table regions exceed %u", who, q.p.n_keys, kMaxKeys);
    // largest batch the workspace holds
    uint64_t batch = (N + kTile - 1) / kTile * kTile;
    const uint64_t cap = max_batch(d, q.p);
    if (batch > cap) batch = cap;
    while (batch > kTile && make_layout(d, q.p, batch).total > ws_bytes) batch = (batch / 2 + kTile - 1) / kTile * kTile;
    q.L = make_layout(d, q.p, batch);
    if (q.L.total > ws_bytes)
        return dg::fail(DG_ERR_WORKSPACE, "%s: workspace %zu bytes cannot hold one tile (%zu needed)", who, ws_bytes, q.L.total);
    char *base = static_cast<char *>(ws);
    q.rows = reinterpret_cast<uint32_t *>(base + q.L.rows);
    q.totals = reinterpret_cast<uint32_t *>(base + q.L.totals);
    q.binbase = reinterpret_cast<uint32_t *>(base + q.L.binbase);
    q.blkbase = reinterpret_cast<uint32_t *>(base + q.L.blkbase);
    q.queue = reinterpret_cast<uint4 *>(base + q.L.queue);
    q.narrow = q.p.max_bins <= 64;                 // then n_keys <= 64 * DG_MAX_LEVELS
    q.grid = sweep_grid(q.p);                      // persistent workgroups of the count and fill sweeps (same tiling)
    return DG_OK;
}

// count sweep and scans of samples [n0, n0 + nb): every workgroup's slice of every bin's queue, the bins' queue ranges,
// the accumulate workgroups per bin; also clears the slot of the batch's largest magnitude
void launch_count(const Prepared &q, const dg_grid_desc *d, const float *u, uint64_t n0, uint64_t nb, hipStream_t st)
{
    const Plan &p = q.p;
    count_lds_kernel<<<q.grid, q.narrow ? kTile : kRingThreads, p.n_keys * 4, st>>>(*d, p, u, n0, nb, q.rows);
    scan_rows_kernel<<<(p.n_keys + kScanKeys - 1) / kScanKeys, kScanKeys * kScanGroups, 0, st>>>(q.rows, q.grid, p.n_keys, slice_round(p), q.totals);
    scan_totals_kernel<<<1, 1024, 0, st>>>(q.totals, p.n_keys, q.binbase, q.blkbase);
}

}  // namespace

int encode_bwd_binned_count(const dg_grid_desc *d, const float *u, uint64_t N, void *ws, size_t ws_bytes, hipStream_t st)
{
    const char *who = "dg_hashgrid_encode_bwd_count";
    Prepared q;
    if (int rc = prepare(who, d, N, ws, ws_bytes, q)) return rc;
    if (q.p.n_keys == 0) return DG_OK;
    if (q.L.batch < N)
        return fail(DG_ERR_WORKSPACE, "%s: counting ahead needs a workspace that holds all %llu samples in one batch (it holds %llu)", who,
                    (unsigned long long)N, (unsigned long long)q.L.batch);
    launch_count(q, d, u, 0, N, st);
    return launch_status(who);
}

int encode_bwd_binned(const dg_grid_desc *d, const float *u, const float *dfeat, uint64_t N, float *dtable, void *ws,
                      size_t ws_bytes, bool counted, hipStream_t st)
{
    const char *who = "dg_hashgrid_encode_bwd";
    Prepared q;
    if (int rc = prepare(who, d, N, ws, ws_bytes, q)) return rc;
    const Plan &p = q.p;
    if (counted && p.n_keys && q.L.batch < N)
        return fail(DG_ERR_WORKSPACE, "%s: the workspace holds %llu of %llu samples: no counts from dg_hashgrid_encode_bwd_count can be in it",
                    who, (unsigned long long)q.L.batch, (unsigned long long)N);
    if (p.first_level > 0) {
        const uint64_t tiles = (N + kCoarseBlock - 1) / kCoarseBlock;
        const uint32_t grid = (uint32_t)(tiles < kCoarseGrid ? tiles : kCoarseGrid);
        coarse_kernel<<<grid, kCoarseBlock, 2 * d->offset[p.first_level] * sizeof(double), st>>>(
            *d, p.first_level, u, (const float2 *)dfeat, N, dtable);
    }
    if (p.n_keys == 0) return launch_status(who);
    const uint64_t batch = q.L.batch;
    for (uint64_t n0 = 0; n0 < N; n0 += batch) {
        const uint64_t nb = N - n0 < batch ? N - n0 : batch;
        if (!counted) launch_count(q, d, u, n0, nb, st);
        if (q.narrow)
            fill_narrow_kernel<<<kBinGrid, kNarrowThreads, kNarrowLds, st>>>(*d, p, u, (const float2 *)dfeat, N, n0, nb, q.rows, q.binbase, q.queue,
                                                                             dtable, q.binbase + p.n_keys + 1);
        else
            fill_ring_kernel<<<q.grid, kRingThreads, p.max_bins * (kRingSlots * 16 + 12) + 16, st>>>(*d, p, u, (const float2 *)dfeat, N, n0, nb, q.rows,
                                                                                                    q.binbase, q.queue, dtable, q.binbase + p.n_keys + 1);
        const uint64_t records = nb * 4ull * (d->n_levels - p.first_level) + slice_padding(p);
        const uint32_t acc_grid = (uint32_t)(records / kAccRecords) + p.n_keys;       // upper bound of the workgroups needed
        accumulate_kernel<<<acc_grid, kAccBlock, 2 * kChunk * sizeof(double), st>>>(*d, p, q.binbase, q.blkbase, (const u32x4 *)q.queue, dtable);
    }
    return launch_status(who);
}

}  // namespace dg
