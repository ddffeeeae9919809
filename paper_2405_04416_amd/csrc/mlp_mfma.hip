// Field MLPs on the matrix cores (v_mfma_f32_32x32x16_f16) for the 32 -> 64 -> 16 density net and
// the (16 + 16) -> 64 -> 64 -> 3 colour net (Sec. 3.2; activations and output clip of Sec. 5.1).
//
// One wavefront owns a tile of 32 samples and keeps every activation of the tile in registers.
// Layers are evaluated transposed, out^T = W . in^T: the weight matrix is the A operand (rows = output
// features), the activations are the B operand (columns = samples).  The result tile then has the
// sample on the lane and the features on the registers, which is again a B operand for the next
// layer once the registers are rounded to fp16 and packed -- the feature order this produces is
// baked into the weight images, so layers chain with no data movement.
//
// Operand and result layouts (lane = 32 h + c, element j / register r):
//   A[row c][k = 8 h + j]     B[k = 8 h + j][col c]     D[row 8 (r / 4) + 4 h + r % 4][col c]
// "Images" are weight tiles pre-arranged in LDS so that one 16-byte read per lane yields an operand.
//
// Backward recomputes the forward, then walks the chain back.  Weight gradients contract over the
// samples, so they need each (delta, activation) pair with the samples on the k axis; a product with
// a 0/1 selection matrix on the matrix cores transposes a tile exactly (fp16 values times one,
// summed with zeros).  Every wavefront accumulates its share of dW in registers over all its tiles,
// writes it to the workspace once, and a second kernel folds the shares in a fixed order.
//
// Appearance features (Sec. 4.4.3: a fixed per-image vector of 16 or 48 values as extra colour-net inputs) widen the
// first colour layer to 48 or 80 inputs.  Forward: NA / 16 more k-steps from a second row table.  Backward: the
// features are constant along a row of samples, so the gradient of their weight columns is
// sum_rows (sum of delta over the row's samples) x (row's features): the per-row delta sums come from one more
// matrix-core product of the transposed delta tile with a 0/1 sample-to-row matrix and are added into a [rows, 64]
// buffer; a small kernel contracts that buffer with the feature rows.  No accumulator registers are added.
#include "dg_internal.h"

namespace dg_mlp_mfma {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef float f16v __attribute__((ext_vector_type(16)));

constexpr int NF = 32, HD = 64, NG = 16, ND = 16, HC = 64, CI = NG + ND;
constexpr int oWd1 = 0, oWd2 = oWd1 + HD * NF, oWc1 = oWd2 + NG * HD, oWc2 = oWc1 + HC * CI, oWc3 = oWc2 + HC * HC;
constexpr int kTotal = oWc3 + 3 * HC;

// image chunks (1 KB each: 64 lanes x 8 halves)
constexpr int cD1 = 0, cD2 = 4, cC1 = 8, cC2 = 12, cC3 = 20, kFwdChunks = 24;
constexpr int cC3T = 24, cC2T = 26, cC1T = 34, cD2T = 38, cD1T = 40, cSelT = 44, cSelN = 46, kAllChunks = 48;

constexpr int kBlock = 256;
constexpr int kWavesPerBlock = kBlock / 64;

// feature held by slot j of lane half h in k-step ks
__device__ __forceinline__ int feat_tiled(int ks, int h, int j) { return 32 * (ks >> 1) + 8 * (2 * (ks & 1) + (j >> 2)) + 4 * h + (j & 3); }
__device__ __forceinline__ int feat_natural(int ks, int h, int j) { return 16 * ks + 8 * h + j; }

// kind: 0 tiled, 1 natural, 2 colour-net input (k-step 0 tiled geometry, k-step 1 natural direction)
__device__ __forceinline__ int feat_of(int kind, int ks, int h, int j)
{
    if (kind == 0) return feat_tiled(ks, h, j);
    if (kind == 1) return feat_natural(ks, h, j);
    return ks == 0 ? feat_tiled(0, h, j) : feat_natural(1, h, j);
}

// A-operand image of a weight matrix W[n_out][n_in] (row-major): rows = outputs (transpose == false)
// or rows = inputs (transpose == true, for the data gradient)
__device__ void build_image(__half *img, const __half *W, int n_out, int n_in, int rows_real, int k_real,
                            int n_mt, int n_ks, int kind, bool transpose)
{
    for (int idx = threadIdx.x; idx < n_mt * n_ks * 512; idx += kBlock) {
        const int j = idx & 7, lane = (idx >> 3) & 63, chunk = idx >> 9;
        const int ks = chunk % n_ks, mt = chunk / n_ks;
        const int row = 32 * mt + (lane & 31), k = feat_of(kind, ks, lane >> 5, j);
        __half v = __float2half(0.0f);
        if (row < rows_real && k < k_real) v = transpose ? W[k * n_in + row] : W[row * n_in + k];
        img[idx] = v;
    }
    (void)n_out;
}

__device__ void build_selection(__half *img, int kind)
{
    for (int idx = threadIdx.x; idx < 2 * 512; idx += kBlock) {
        const int j = idx & 7, lane = (idx >> 3) & 63, p = idx >> 9;
        const int f = (kind == 0 ? feat_tiled(p, lane >> 5, j) : feat_natural(p, lane >> 5, j)) & 31;
        img[idx] = __float2half(f == (lane & 31) ? 1.0f : 0.0f);
    }
}

__device__ void build_forward_images(__half *lds, const __half *w)
{
    build_image(lds + cD1 * 512, w + oWd1, HD, NF, HD, NF, 2, 2, 1, false);
    build_image(lds + cD2 * 512, w + oWd2, NG, HD, NG, HD, 1, 4, 0, false);
    build_image(lds + cC1 * 512, w + oWc1, HC, CI, HC, CI, 2, 2, 2, false);
    build_image(lds + cC2 * 512, w + oWc2, HC, HC, HC, HC, 2, 4, 0, false);
    build_image(lds + cC3 * 512, w + oWc3, 3, HC, 3, HC, 1, 4, 0, false);
}

__device__ void build_backward_images(__half *lds, const __half *w)
{
    build_image(lds + cC3T * 512, w + oWc3, 3, HC, HC, 3, 2, 1, 0, true);
    build_image(lds + cC2T * 512, w + oWc2, HC, HC, HC, HC, 2, 4, 0, true);
    build_image(lds + cC1T * 512, w + oWc1, HC, CI, NG, HC, 1, 4, 0, true);     // direction inputs get no gradient
    build_image(lds + cD2T * 512, w + oWd2, NG, HD, HD, NG, 2, 1, 0, true);
    build_image(lds + cD1T * 512, w + oWd1, HD, NF, NF, HD, 1, 4, 0, true);
    build_selection(lds + cSelT * 512, 0);
    build_selection(lds + cSelN * 512, 1);
}

__device__ __forceinline__ h8 image(const __half *lds, int chunk, int lane)
{
    return reinterpret_cast<const h8 *>(lds)[chunk * 64 + lane];
}

// Returns its argument, in a way the compiler cannot see through: LDS reads indexed with the result are
// issued where they are used, not hoisted out of the tile loop and held in registers for its whole length.
__device__ __forceinline__ int opaque(int x)
{
    asm volatile("" : "+v"(x));
    return x;
}

__device__ __forceinline__ f16v mma(h8 a, h8 b, f16v c) { return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0); }

__device__ __forceinline__ f16v zero16()
{
    f16v z;
#pragma unroll
    for (int i = 0; i < 16; ++i) z[i] = 0.0f;
    return z;
}

__device__ __forceinline__ float fast_sigmoid(float x)
{
    return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * x));
}
__device__ __forceinline__ float clip15(float x) { return fminf(fmaxf(x, -15.0f), 15.0f); }

// max(x, 0) on four pairs of halves, one instruction per pair
__device__ __forceinline__ h8 relu_pairs(h8 x)
{
    typedef uint32_t u4 __attribute__((ext_vector_type(4)));
    u4 w = __builtin_bit_cast(u4, x);
#pragma unroll
    for (int i = 0; i < 4; ++i) asm("v_pk_max_f16 %0, %1, 0" : "=v"(w[i]) : "v"(w[i]));
    return __builtin_bit_cast(h8, w);
}

// registers 8p .. 8p+7 of a result tile, activated, rounded to fp16 and packed: k-step (m, p) of the next operand
template <int ACT>   // 0 identity, 1 ReLU, 2 sigmoid
__device__ __forceinline__ h8 pack_half(const f16v &c, int p)
{
    h8 out;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        float v = c[8 * p + j];
        if (ACT == 2) v = fast_sigmoid(v);
        out[j] = (_Float16)v;
    }
    // ReLU after the rounding gives the same values as before it (rounding is monotone and keeps 0) and works on pairs
    if (ACT == 1) out = relu_pairs(out);
    return out;
}

struct Tile {
    h8 x0[2], h1[4], xc[2], xa[3], c1[4], c2[4];      // xa: appearance inputs (unused without them)
    float geo0, sigma, raw[3], rgb[3];     // meaningful on lanes with h == 0
};

// NA: appearance inputs (0, 16 or 48); their weight images start at chunk c_app
template <int NA>
__device__ __forceinline__ void forward_tile(const __half *lds, int lane, uint32_t act_c, Tile &t, int c_app = 0)
{
    f16v acc[2];
    // density layer 1: 32 -> 64, ReLU
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
        acc[mt] = zero16();
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) acc[mt] = mma(image(lds, cD1 + mt * 2 + ks, lane), t.x0[ks], acc[mt]);
    }
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) t.h1[ks] = pack_half<1>(acc[ks >> 1], ks & 1);
    // density layer 2: 64 -> 16, raw
    f16v geo = zero16();
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) geo = mma(image(lds, cD2 + ks, lane), t.h1[ks], geo);
    t.geo0 = geo[0];
    t.sigma = __expf(clip15(geo[0]));
    t.xc[0] = pack_half<0>(geo, 0);
    // colour layer 1: (16 + 16) -> 64
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
        acc[mt] = zero16();
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) acc[mt] = mma(image(lds, cC1 + mt * 2 + ks, lane), t.xc[ks], acc[mt]);
#pragma unroll
        for (int ks = 0; ks < NA / 16; ++ks) acc[mt] = mma(image(lds, c_app + mt * (NA / 16) + ks, lane), t.xa[ks], acc[mt]);
    }
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) t.c1[ks] = act_c ? pack_half<2>(acc[ks >> 1], ks & 1) : pack_half<1>(acc[ks >> 1], ks & 1);
    // colour layer 2: 64 -> 64
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
        acc[mt] = zero16();
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) acc[mt] = mma(image(lds, cC2 + mt * 4 + ks, lane), t.c1[ks], acc[mt]);
    }
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) t.c2[ks] = act_c ? pack_half<2>(acc[ks >> 1], ks & 1) : pack_half<1>(acc[ks >> 1], ks & 1);
    // colour layer 3: 64 -> 3, raw
    f16v out = zero16();
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) out = mma(image(lds, cC3 + ks, lane), t.c2[ks], out);
#pragma unroll
    for (int c = 0; c < 3; ++c) { t.raw[c] = out[c]; t.rgb[c] = fast_sigmoid(clip15(out[c])); }
}

// features arrive as level-major planes [16][n_samples] of half2; slot j of k-step ks on lane half h
// is feature 16 ks + 8 h + j, i.e. component j % 2 of level 8 ks + 4 h + j / 2
template <int NA>
__device__ __forceinline__ void load_inputs(const __half *feat, const __half *dir_enc, const __half *app, uint32_t S,
                                            uint64_t n_samples, uint64_t n, bool valid, int h, Tile &t)
{
    const h8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
    if (valid) {
        typedef uint32_t u4 __attribute__((ext_vector_type(4)));
        const uint32_t *planes = reinterpret_cast<const uint32_t *>(feat);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            u4 bits;
#pragma unroll
            for (int q = 0; q < 4; ++q) bits[q] = planes[(size_t)(8 * ks + 4 * h + q) * n_samples + n];
            t.x0[ks] = __builtin_bit_cast(h8, bits);
        }
        t.xc[1] = reinterpret_cast<const h8 *>(dir_enc + (n / S) * ND)[h];
#pragma unroll
        for (int ks = 0; ks < NA / 16; ++ks) t.xa[ks] = reinterpret_cast<const h8 *>(app + (n / S) * NA)[2 * ks + h];
    } else {
        t.x0[0] = zero; t.x0[1] = zero; t.xc[1] = zero;
#pragma unroll
        for (int ks = 0; ks < NA / 16; ++ks) t.xa[ks] = zero;
    }
}

template <int NA>
__global__ void __launch_bounds__(kBlock, 4)
fwd_kernel(const __half *__restrict__ weights, const __half *__restrict__ feat, const __half *__restrict__ dir_enc,
           const __half *__restrict__ app, uint32_t S, uint64_t n_samples, uint32_t act_c, float *__restrict__ sigma,
           float *__restrict__ rgb)
{
    __shared__ __attribute__((aligned(16))) __half lds[(kFwdChunks + 2 * (NA / 16)) * 512];
    build_forward_images(lds, weights);
    if (NA > 0) build_image(lds + kFwdChunks * 512, weights + kTotal, HC, NA, HC, NA, 2, NA / 16, 1, false);
    __syncthreads();
    const int lane = threadIdx.x & 63, h = lane >> 5;
    const uint64_t n_tiles = (n_samples + 31) / 32;
    const uint64_t wave = (uint64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
    const uint64_t n_waves = (uint64_t)gridDim.x * kWavesPerBlock;
    for (uint64_t tile = wave; tile < n_tiles; tile += n_waves) {
        const uint64_t n = tile * 32 + (lane & 31);
        const bool valid = n < n_samples;
        Tile t;
        load_inputs<NA>(feat, dir_enc, app, S, n_samples, n, valid, h, t);
        forward_tile<NA>(lds, opaque(lane), act_c, t, kFwdChunks);
        if (valid && h == 0) {
            sigma[n] = t.sigma;
            rgb[3 * n] = t.rgb[0]; rgb[3 * n + 1] = t.rgb[1]; rgb[3 * n + 2] = t.rgb[2];
        }
    }
}

// ---------------------------------------------------------------------------------------- evaluation rendering, fused
// Forward-only rendering (Sec. 4.4.2: every sub-model renders its segments, the partial colour, depth and transmittance
// are merged afterwards): the field networks and the local volume rendering (Eq. 3) of one segment in one wavefront.
// A segment of S <= 64 samples is two tiles of the forward above (samples 0..31 and 32..S-1); their densities and
// colours end up on lanes 0..31, the second tile's are moved to lanes 32..63, and the front-to-back product over the
// 64 lanes is a prefix scan -- sigma and rgb never leave the registers.  The arithmetic of the scan is that of the
// separate compositing kernels (alpha from expm1, transmittance as a running product of exp(-sigma delta)).
__device__ __forceinline__ float wave_inclusive_product(float v, int lane)
{
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const float up = __shfl_up(v, off, 64);
        if (lane >= off) v *= up;
    }
    return v;
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

template <int NA>
__global__ void __launch_bounds__(kBlock, 4)
render_fwd_kernel(const __half *__restrict__ weights, const __half *__restrict__ feat, const __half *__restrict__ dir_enc,
                  const __half *__restrict__ app, uint32_t S, uint32_t n_seg, uint32_t act_c, const float *__restrict__ delta,
                  const float *__restrict__ t_samples, const uint32_t *__restrict__ seg_ray, const uint32_t *__restrict__ seg_slot,
                  uint32_t k_max, float *__restrict__ Ck, float *__restrict__ Tk, float *__restrict__ Dk)
{
    __shared__ __attribute__((aligned(16))) __half lds[(kFwdChunks + 2 * (NA / 16)) * 512];
    build_forward_images(lds, weights);
    if (NA > 0) build_image(lds + kFwdChunks * 512, weights + kTotal, HC, NA, HC, NA, 2, NA / 16, 1, false);
    __syncthreads();
    const int lane = threadIdx.x & 63, h = lane >> 5;
    const uint64_t n_samples = (uint64_t)n_seg * S;
    const uint32_t wave = blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6), n_waves = gridDim.x * kWavesPerBlock;
    for (uint32_t seg = wave; seg < n_seg; seg += n_waves) {
        const uint64_t first = (uint64_t)seg * S;
        float sig[2], col[2][3];
#pragma unroll
        for (int part = 0; part < 2; ++part) {
            const uint32_t s = 32u * part + (lane & 31);
            const bool valid = s < S;
            Tile t;
            load_inputs<NA>(feat, dir_enc, app, S, n_samples, first + (valid ? s : 0), valid, h, t);
            forward_tile<NA>(lds, opaque(lane), act_c, t, kFwdChunks);
            sig[part] = t.sigma;
            col[part][0] = t.rgb[0]; col[part][1] = t.rgb[1]; col[part][2] = t.rgb[2];
        }
        // sample `lane` of the segment: first tile on lanes 0..31 as it stands, second tile fetched from lanes 0..31
        // (every lane takes part in the exchange; the choice comes afterwards: a lane must not read from lanes that a
        // branch has switched off)
        const float s_up = __shfl(sig[1], lane & 31, 64), a_up = __shfl(col[1][0], lane & 31, 64);
        const float b_up = __shfl(col[1][1], lane & 31, 64), c_up = __shfl(col[1][2], lane & 31, 64);
        const float sigma_s = h ? s_up : sig[0], r0 = h ? a_up : col[0][0], r1 = h ? b_up : col[0][1], r2 = h ? c_up : col[0][2];
        const bool live = (uint32_t)lane < S;
        const uint64_t n = first + (live ? lane : 0);
        const float x = live ? sigma_s * delta[n] : 0.0f;
        const float incl = wave_inclusive_product(expf(-x), lane);
        float before = __shfl_up(incl, 1, 64);
        if (lane == 0) before = 1.0f;
        const float wgt = live ? before * -expm1f(-x) : 0.0f;
        const float c0 = wave_sum(wgt * r0), c1 = wave_sum(wgt * r1), c2 = wave_sum(wgt * r2);
        const float depth = t_samples ? wave_sum(live ? wgt * t_samples[n] : 0.0f) : 0.0f;
        const float trans = __shfl(incl, 63, 64);
        if (lane == 0) {
            const size_t dst = (size_t)seg_ray[seg] * k_max + seg_slot[seg];
            Ck[3 * dst] = c0; Ck[3 * dst + 1] = c1; Ck[3 * dst + 2] = c2;
            Tk[dst] = trans;
            if (Dk) Dk[dst] = depth;
        }
    }
}

// ---------------------------------------------------------------------------------------- backward

// transpose of one 32-feature tile of a packed tensor: x0 / x1 are the two k-steps that hold the tile,
// sel0 / sel1 the matching selection images; result: the two sample k-steps of the transposed tile
__device__ __forceinline__ void transpose_tile(h8 x0, h8 x1, h8 sel0, h8 sel1, h8 out[2])
{
    f16v c = zero16();
    c = mma(x0, sel0, c);
    c = mma(x1, sel1, c);
    out[0] = pack_half<0>(c, 0);
    out[1] = pack_half<0>(c, 1);
}
__device__ __forceinline__ void transpose_half_tile(h8 x0, h8 sel0, h8 out[2])
{
    f16v c = zero16();
    c = mma(x0, sel0, c);
    out[0] = pack_half<0>(c, 0);
    out[1] = pack_half<0>(c, 1);
}

// delta = fp16(g * act'(a)) for one k-step; a is the packed (rounded) activation
template <int ACT>   // 1 ReLU, 2 sigmoid
__device__ __forceinline__ h8 delta_from(const f16v &g, int p, h8 a)
{
    h8 out;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const float av = (float)a[j];
        const float d = ACT == 2 ? av * (1.0f - av) : (av > 0.0f ? 1.0f : 0.0f);
        out[j] = (_Float16)(g[8 * p + j] * d);
    }
    return out;
}

__device__ __forceinline__ void store_share(float *dst, int n_in, int rows_real, int ot, int it, int lane, const f16v &acc)
{
    const int h = lane >> 5, i = 32 * it + (lane & 31);
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int o = 32 * ot + 8 * (r >> 2) + 4 * h + (r & 3);
        if (o < rows_real) dst[o * n_in + i] = acc[r];
    }
}

// The backward pass runs as two kernels so that neither has to hold all twelve dW tiles (192
// accumulator registers) next to the activations:
//   colour_bwd : recomputes the whole forward, back-propagates the colour net, accumulates dWc1..3
//                (8 tiles = 128 registers; the weight images are re-read from LDS tile by tile so that
//                the rest fits the 256 registers of two wavefronts per SIMD, which keeps every MFMA
//                result in ordinary registers) and leaves delta_geo (gradient of the 16 density outputs, sigma term included,
//                already scaled and rounded to fp16, in operand order) in the workspace;
//   density_bwd: recomputes the density hidden layer, back-propagates it from delta_geo, accumulates
//                dWd1..2 and writes the feature gradient planes.
template <int NA>
__global__ void __launch_bounds__(kBlock, 2)
colour_bwd_kernel(const __half *__restrict__ weights, const __half *__restrict__ feat, const __half *__restrict__ dir_enc,
                  const __half *__restrict__ app, uint32_t S, uint64_t n_samples, uint32_t act_c,
                  const float *__restrict__ dsigma, const float *__restrict__ drgb, float loss_scale, h8 *__restrict__ dgeo,
                  float *__restrict__ shares, float *__restrict__ row_delta)
{
    __shared__ __attribute__((aligned(16))) __half lds[(kAllChunks + 2 * (NA / 16)) * 512];
    __shared__ float acc3[kWavesPerBlock * 2 * 3 * 32];
    build_forward_images(lds, weights);
    build_backward_images(lds, weights);
    if (NA > 0) build_image(lds + kAllChunks * 512, weights + kTotal, HC, NA, HC, NA, 2, NA / 16, 1, false);
    __syncthreads();
    const int lane_fixed = threadIdx.x & 63, h = lane_fixed >> 5;
    const uint64_t n_tiles = (n_samples + 31) / 32;
    const uint64_t wave = (uint64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
    const uint64_t n_waves = (uint64_t)gridDim.x * kWavesPerBlock;
    const h8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};

    f16v gWc2[2][2], gWc1[2];               // [output tile][input tile]
#pragma unroll
    for (int a = 0; a < 2; ++a) { gWc1[a] = zero16(); gWc2[a][0] = zero16(); gWc2[a][1] = zero16(); }
    // The output layer has 3 rows: its gradient tiles are 3 real rows of 32, too little to deserve 32 accumulator
    // registers next to the others.  Each wavefront keeps those 3 x 64 sums in LDS words of its own (one owner lane
    // per word, plain read-add-write, so the order of the additions is fixed).
    float *gWc3 = acc3 + (threadIdx.x >> 6) * (2 * 3 * 32);      // [input tile][row][column]
    if (h == 0) {
#pragma unroll
        for (int k = 0; k < 6; ++k) gWc3[k * 32 + (lane_fixed & 31)] = 0.0f;
    }

    for (uint64_t tile = wave; tile < n_tiles; tile += n_waves) {
        const uint64_t n = tile * 32 + (lane_fixed & 31);
        const bool valid = n < n_samples;
        const int lane = opaque(lane_fixed);
        Tile t;
        load_inputs<NA>(feat, dir_enc, app, S, n_samples, n, valid, h, t);
        float ds = 0.0f, dc[3] = {0.0f, 0.0f, 0.0f};
        if (valid && h == 0) {                 // issued before the forward so the latency hides behind it
            ds = dsigma[n];
            dc[0] = drgb[3 * n]; dc[1] = drgb[3 * n + 1]; dc[2] = drgb[3 * n + 2];
        }
        forward_tile<NA>(lds, lane, act_c, t, kAllChunks);
        const h8 selT0 = image(lds, cSelT, lane), selT1 = image(lds, cSelT + 1, lane);

        // ---- output layer of the colour net
        h8 d3 = zero8;
        if (valid && h == 0) {
#pragma unroll
            for (int c = 0; c < 3; ++c) {
                const bool pass = t.raw[c] >= -15.0f && t.raw[c] <= 15.0f;
                d3[c] = (_Float16)(pass ? loss_scale * dc[c] * t.rgb[c] * (1.0f - t.rgb[c]) : 0.0f);
            }
        }
        h8 td[2][2], ta[2][2];      // transposed delta / activation: [feature tile][sample k-step]
        transpose_half_tile(d3, selT0, td[0]);
        transpose_tile(t.c2[0], t.c2[1], selT0, selT1, ta[0]);
        transpose_tile(t.c2[2], t.c2[3], selT0, selT1, ta[1]);
#pragma unroll
        for (int it = 0; it < 2; ++it) {
            f16v part = mma(td[0][0], ta[it][0], zero16());
            part = mma(td[0][1], ta[it][1], part);
            if (h == 0) {                  // rows 0..2 of the tile are registers 0..2 of the lower half's lanes
#pragma unroll
                for (int o = 0; o < 3; ++o) gWc3[(it * 3 + o) * 32 + (lane_fixed & 31)] += part[o];
            }
        }
        f16v g[2];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) g[mt] = mma(image(lds, cC3T + mt, lane), d3, zero16());

        // ---- second hidden layer of the colour net
        h8 dl[4];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) dl[ks] = act_c ? delta_from<2>(g[ks >> 1], ks & 1, t.c2[ks]) : delta_from<1>(g[ks >> 1], ks & 1, t.c2[ks]);
        transpose_tile(dl[0], dl[1], selT0, selT1, td[0]);
        transpose_tile(dl[2], dl[3], selT0, selT1, td[1]);
        transpose_tile(t.c1[0], t.c1[1], selT0, selT1, ta[0]);
        transpose_tile(t.c1[2], t.c1[3], selT0, selT1, ta[1]);
#pragma unroll
        for (int ot = 0; ot < 2; ++ot)
#pragma unroll
            for (int it = 0; it < 2; ++it)
#pragma unroll
                for (int p = 0; p < 2; ++p) gWc2[ot][it] = mma(td[ot][p], ta[it][p], gWc2[ot][it]);
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            g[mt] = zero16();
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) g[mt] = mma(image(lds, cC2T + mt * 4 + ks, lane), dl[ks], g[mt]);
        }

        // ---- first hidden layer of the colour net
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) dl[ks] = act_c ? delta_from<2>(g[ks >> 1], ks & 1, t.c1[ks]) : delta_from<1>(g[ks >> 1], ks & 1, t.c1[ks]);
        transpose_tile(dl[0], dl[1], selT0, selT1, td[0]);
        transpose_tile(dl[2], dl[3], selT0, selT1, td[1]);
        transpose_tile(t.xc[0], t.xc[1], selT0, image(lds, cSelN + 1, lane), ta[0]);
#pragma unroll
        for (int ot = 0; ot < 2; ++ot)
#pragma unroll
            for (int p = 0; p < 2; ++p) gWc1[ot] = mma(td[ot][p], ta[0][p], gWc1[ot]);
        if (NA > 0) {
            // per-row sums of delta for the appearance columns: delta^T (features x samples) times the 0/1 matrix
            // "sample s lies in the tile's local row c"; column c of the result is the sum over that row's samples
            const uint64_t n0 = tile * 32;
            const uint64_t row0 = n0 / S;                                             // row of the tile's first sample
            const uint32_t rem0 = (uint32_t)(n0 - row0 * S), c = lane_fixed & 31;
            // local row of sample s of the tile: rows of 32 or more samples change at most once, at sample `turn`;
            // shorter rows: (rem0 + s) / S on integers below 64, exact through a float reciprocal
            const bool wide = S >= 32;
            const uint32_t turn = S - rem0;
            const float inv_S = 1.0f / (float)S;
            auto local_row = [&](uint32_t smp) {
                return wide ? (smp >= turn ? 1u : 0u) : (uint32_t)((float)(rem0 + smp) * inv_S + 1e-3f);
            };
            const uint32_t last = (uint32_t)(n_samples - 1 - n0 < 31 ? n_samples - 1 - n0 : 31);
            const uint32_t n_local = local_row(last) + 1u;                            // rows with samples in this tile
            h8 in_row[2];
#pragma unroll
            for (int p = 0; p < 2; ++p)
#pragma unroll
                for (int j = 0; j < 8; ++j)      // slot j of k-step p holds sample feat_tiled(p, h, j) of the tile, as in td
                    in_row[p][j] = (_Float16)(local_row((uint32_t)feat_tiled(p, h, j)) == c ? 1.0f : 0.0f);
#pragma unroll
            for (int ot = 0; ot < 2; ++ot) {
                f16v sums = mma(td[ot][0], in_row[0], zero16());
                sums = mma(td[ot][1], in_row[1], sums);
                if (c < n_local) {
                    float *dst = row_delta + (row0 + c) * HC + 32 * ot + 4 * h;
#pragma unroll
                    for (int r = 0; r < 16; ++r) unsafeAtomicAdd(dst + 8 * (r >> 2) + (r & 3), sums[r]);
                }
            }
        }
        f16v gx = zero16();
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) gx = mma(image(lds, cC1T + ks, lane), dl[ks], gx);

        // ---- density net output: geometry features feed the colour net, output 0 also feeds exp()
        if (valid && h == 0) {
            const bool pass0 = t.geo0 >= -15.0f && t.geo0 <= 15.0f;
            gx[0] += pass0 ? loss_scale * ds * t.sigma : 0.0f;
        }
        if (valid) dgeo[2 * n + h] = pack_half<0>(gx, 0);
    }

    float *mine = shares + wave * (kTotal - oWc1) - oWc1;       // colour shares hold elements [oWc1, kTotal)
    const int lane = lane_fixed;
    if (h == 0) {
#pragma unroll
        for (int it = 0; it < 2; ++it)
#pragma unroll
            for (int o = 0; o < 3; ++o) mine[oWc3 + o * HC + 32 * it + (lane & 31)] = gWc3[(it * 3 + o) * 32 + (lane & 31)];
    }
#pragma unroll
    for (int ot = 0; ot < 2; ++ot) {
        store_share(mine + oWc2, HC, HC, ot, 0, lane, gWc2[ot][0]);
        store_share(mine + oWc2, HC, HC, ot, 1, lane, gWc2[ot][1]);
        store_share(mine + oWc1, CI, HC, ot, 0, lane, gWc1[ot]);
    }
}

__global__ void __launch_bounds__(kBlock, 2)
density_bwd_kernel(const __half *__restrict__ weights, const __half *__restrict__ feat, uint64_t n_samples,
                   const h8 *__restrict__ dgeo, float loss_scale, float *__restrict__ dfeat, float *__restrict__ shares)
{
    // images: density layer 1 forward (4 chunks), Wd2^T (2), Wd1^T (4), selections (4)
    constexpr int kD1 = 0, kD2T = 4, kD1T = 6, kST = 10, kSN = 12, kChunks = 14;
    __shared__ __attribute__((aligned(16))) __half lds[kChunks * 512];
    build_image(lds + kD1 * 512, weights + oWd1, HD, NF, HD, NF, 2, 2, 1, false);
    build_image(lds + kD2T * 512, weights + oWd2, NG, HD, HD, NG, 2, 1, 0, true);
    build_image(lds + kD1T * 512, weights + oWd1, HD, NF, NF, HD, 1, 4, 0, true);
    build_selection(lds + kST * 512, 0);
    build_selection(lds + kSN * 512, 1);
    __syncthreads();
    const int lane = threadIdx.x & 63, h = lane >> 5;
    const uint64_t n_tiles = (n_samples + 31) / 32;
    const uint64_t wave = (uint64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
    const uint64_t n_waves = (uint64_t)gridDim.x * kWavesPerBlock;
    const float inv_scale = 1.0f / loss_scale;
    const h8 selT0 = image(lds, kST, lane), selT1 = image(lds, kST + 1, lane);
    const h8 selN0 = image(lds, kSN, lane), selN1 = image(lds, kSN + 1, lane);
    const h8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};

    f16v gWd2[2], gWd1[2];
#pragma unroll
    for (int a = 0; a < 2; ++a) { gWd2[a] = zero16(); gWd1[a] = zero16(); }

    for (uint64_t tile = wave; tile < n_tiles; tile += n_waves) {
        const uint64_t n = tile * 32 + (lane & 31);
        const bool valid = n < n_samples;
        Tile t;
        load_inputs<0>(feat, nullptr, nullptr, 1, n_samples, n, false, h, t);      // zeroes
        if (valid) {
            typedef uint32_t u4 __attribute__((ext_vector_type(4)));
            const uint32_t *planes = reinterpret_cast<const uint32_t *>(feat);
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                u4 bits;
#pragma unroll
                for (int q = 0; q < 4; ++q) bits[q] = planes[(size_t)(8 * ks + 4 * h + q) * n_samples + n];
                t.x0[ks] = __builtin_bit_cast(h8, bits);
            }
        }
        const h8 dg = valid ? dgeo[2 * n + h] : zero8;
        f16v acc[2];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
            acc[mt] = zero16();
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) acc[mt] = mma(image(lds, kD1 + mt * 2 + ks, lane), t.x0[ks], acc[mt]);
        }
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) t.h1[ks] = pack_half<1>(acc[ks >> 1], ks & 1);

        h8 td[2][2], ta[2][2];
        transpose_half_tile(dg, selT0, td[0]);
        transpose_tile(t.h1[0], t.h1[1], selT0, selT1, ta[0]);
        transpose_tile(t.h1[2], t.h1[3], selT0, selT1, ta[1]);
#pragma unroll
        for (int it = 0; it < 2; ++it)
#pragma unroll
            for (int p = 0; p < 2; ++p) gWd2[it] = mma(td[0][p], ta[it][p], gWd2[it]);
        f16v g[2];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) g[mt] = mma(image(lds, kD2T + mt, lane), dg, zero16());

        h8 dl[4];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) dl[ks] = delta_from<1>(g[ks >> 1], ks & 1, t.h1[ks]);
        transpose_tile(dl[0], dl[1], selT0, selT1, td[0]);
        transpose_tile(dl[2], dl[3], selT0, selT1, td[1]);
        transpose_tile(t.x0[0], t.x0[1], selN0, selN1, ta[0]);
#pragma unroll
        for (int ot = 0; ot < 2; ++ot)
#pragma unroll
            for (int p = 0; p < 2; ++p) gWd1[ot] = mma(td[ot][p], ta[0][p], gWd1[ot]);
        f16v gf = zero16();
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) gf = mma(image(lds, kD1T + ks, lane), dl[ks], gf);
        if (valid) {
            // registers 4q .. 4q+3 hold features 8q + 4h .. + 3: levels 4q + 2h and 4q + 2h + 1 of the planes [16][n_samples][2]
            float2 *planes = reinterpret_cast<float2 *>(dfeat);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                planes[(size_t)(4 * q + 2 * h) * n_samples + n] = make_float2(gf[4 * q] * inv_scale, gf[4 * q + 1] * inv_scale);
                planes[(size_t)(4 * q + 2 * h + 1) * n_samples + n] = make_float2(gf[4 * q + 2] * inv_scale, gf[4 * q + 3] * inv_scale);
            }
        }
    }

    float *mine = shares + wave * oWc1;                         // density shares hold elements [0, oWc1)
#pragma unroll
    for (int ot = 0; ot < 2; ++ot) store_share(mine + oWd1, NF, HD, ot, 0, lane, gWd1[ot]);
    store_share(mine + oWd2, HD, NG, 0, 0, lane, gWd2[0]);
    store_share(mine + oWd2, HD, NG, 0, 1, lane, gWd2[1]);
}

// dW[e] += (sum of the wavefronts' shares of element e) / loss_scale, in a fixed order.  Elements below
// oWc1 (density net) come from density_shares [n_d][oWc1], the rest from colour_shares [n_c][kTotal - oWc1].
// A workgroup serves 64 consecutive elements; 16 groups of threads each sum every 16th share, then the 16
// partial sums are added in a fixed order.
constexpr int kFoldElems = 64, kFoldGroups = 16;
static_assert(oWc1 % kFoldElems == 0, "a fold workgroup must not span both share regions");
__global__ void __launch_bounds__(kFoldElems * kFoldGroups)
fold_shares_kernel(const float *__restrict__ density_shares, uint32_t n_d, const float *__restrict__ colour_shares,
                   uint32_t n_c, float inv_scale, float *__restrict__ dW)
{
    __shared__ float part[kFoldGroups][kFoldElems];
    const uint32_t col = threadIdx.x % kFoldElems, group = threadIdx.x / kFoldElems;
    const uint32_t e = blockIdx.x * kFoldElems + col;
    float s0 = 0.0f, s1 = 0.0f;
    if (e < (uint32_t)kTotal) {
        const bool dens = e < (uint32_t)oWc1;
        const float *src = dens ? density_shares + e : colour_shares + (e - oWc1);
        const uint32_t stride = dens ? oWc1 : kTotal - oWc1, n = dens ? n_d : n_c;
        uint32_t b = group;
        for (; b + kFoldGroups < n; b += 2 * kFoldGroups) {
            s0 += src[(size_t)b * stride];
            s1 += src[(size_t)(b + kFoldGroups) * stride];
        }
        if (b < n) s0 += src[(size_t)b * stride];
    }
    part[group][col] = s0 + s1;
    __syncthreads();
    if (group == 0 && e < (uint32_t)kTotal) {
        float s = 0.0f;
#pragma unroll
        for (int k = 0; k < kFoldGroups; ++k) s += part[k][col];
        dW[e] += s * inv_scale;
    }
}

// dW[kTotal + o * NA + a] += inv_scale * sum_rows row_delta[row][o] * app[row][a].  A workgroup of four row groups
// walks rows with a grid stride, eight rows in flight per thread (independent loads); thread (o, quarter q) of a row
// group keeps NA / 4 sums; the groups' sums meet in LDS and the workgroup issues one atomic per weight (atomics on the
// same few thousand addresses serialise, so there are few workgroups).
constexpr int kWgradGroups = 4, kWgradBlock = kWgradGroups * 256, kWgradGrid = 256;
template <int NA>
__global__ void __launch_bounds__(kWgradBlock)
appearance_wgrad_kernel(const float *__restrict__ row_delta, const __half *__restrict__ app, uint64_t n_rows, float inv_scale,
                        float *__restrict__ dW)
{
    constexpr int kPer = NA / 4, kBatch = 8;
    __shared__ float part[kWgradGroups - 1][HC * NA];
    const int o = threadIdx.x & 63, q = (threadIdx.x >> 6) & 3, group = threadIdx.x >> 8;
    float acc[kPer];
#pragma unroll
    for (int a = 0; a < kPer; ++a) acc[a] = 0.0f;
    for (uint64_t first = ((uint64_t)blockIdx.x * kWgradGroups + group) * kBatch; first < n_rows;
         first += (uint64_t)gridDim.x * kWgradGroups * kBatch) {
        float d[kBatch];
        uint2 x[kBatch][kPer / 4];                          // kPer halves = kPer / 4 words of 8 bytes
#pragma unroll
        for (int b = 0; b < kBatch; ++b) {
            const uint64_t row = first + b < n_rows ? first + b : n_rows - 1;
            d[b] = first + b < n_rows ? row_delta[row * HC + o] : 0.0f;
            const uint2 *src = reinterpret_cast<const uint2 *>(app + row * NA + q * kPer);
#pragma unroll
            for (int w = 0; w < kPer / 4; ++w) x[b][w] = src[w];
        }
#pragma unroll
        for (int b = 0; b < kBatch; ++b)
#pragma unroll
            for (int w = 0; w < kPer / 4; ++w) {
                const __half2 lo = __builtin_bit_cast(__half2, x[b][w].x), hi = __builtin_bit_cast(__half2, x[b][w].y);
                acc[4 * w] = __builtin_fmaf(d[b], __low2float(lo), acc[4 * w]);
                acc[4 * w + 1] = __builtin_fmaf(d[b], __high2float(lo), acc[4 * w + 1]);
                acc[4 * w + 2] = __builtin_fmaf(d[b], __low2float(hi), acc[4 * w + 2]);
                acc[4 * w + 3] = __builtin_fmaf(d[b], __high2float(hi), acc[4 * w + 3]);
            }
    }
    if (group > 0) {
#pragma unroll
        for (int a = 0; a < kPer; ++a) part[group - 1][o * NA + q * kPer + a] = acc[a];
    }
    __syncthreads();
    if (group == 0) {
#pragma unroll
        for (int a = 0; a < kPer; ++a) {
            float v = acc[a];
#pragma unroll
            for (int g = 0; g < kWgradGroups - 1; ++g) v += part[g][o * NA + q * kPer + a];
            unsafeAtomicAdd(dW + kTotal + o * NA + q * kPer + a, v * inv_scale);
        }
    }
}

__global__ void __launch_bounds__(kBlock)
zero_kernel(float *__restrict__ p, uint64_t n)
{
    for (uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (uint64_t)gridDim.x * kBlock) p[i] = 0.0f;
}

constexpr uint32_t kGridColour = 512;      // persistent workgroups: two per compute unit of MI355X
constexpr uint32_t kGridDensity = 512;     // the lighter kernel fits two workgroups per compute unit

inline size_t align256(size_t x) { return (x + 255) / 256 * 256; }

}  // namespace dg_mlp_mfma

namespace dg {

size_t mlp_mfma_workspace_bytes(uint64_t N, uint32_t n_app, uint32_t S)
{
    using namespace dg_mlp_mfma;
    const uint64_t n_rows = n_app ? (N + S - 1) / S : 0;
    return align256((size_t)kGridDensity * kWavesPerBlock * oWc1 * sizeof(float)) +
           align256((size_t)kGridColour * kWavesPerBlock * (kTotal - oWc1) * sizeof(float)) + align256((size_t)N * 32) +
           align256((size_t)n_rows * HC * sizeof(float));
}

size_t mlp_mfma_weight_count(uint32_t n_app) { return (size_t)dg_mlp_mfma::kTotal + (size_t)dg_mlp_mfma::HC * n_app; }

void mlp_mfma_fwd(const void *weights, const void *feat, const void *dir_enc, const void *app, uint32_t n_app, uint32_t S,
                  uint64_t N, uint32_t act_c, float *sigma, float *rgb, hipStream_t st)
{
    using namespace dg_mlp_mfma;
    const uint64_t tiles = (N + 31) / 32, blocks_needed = (tiles + kWavesPerBlock - 1) / kWavesPerBlock;
    const uint32_t grid = (uint32_t)(blocks_needed < 2048 ? blocks_needed : 2048);
    const __half *w = (const __half *)weights, *f = (const __half *)feat, *dr = (const __half *)dir_enc, *ap = (const __half *)app;
    if (n_app == 0) fwd_kernel<0><<<grid, kBlock, 0, st>>>(w, f, dr, ap, S, N, act_c, sigma, rgb);
    else if (n_app == 16) fwd_kernel<16><<<grid, kBlock, 0, st>>>(w, f, dr, ap, S, N, act_c, sigma, rgb);
    else fwd_kernel<48><<<grid, kBlock, 0, st>>>(w, f, dr, ap, S, N, act_c, sigma, rgb);
}

void mlp_mfma_render(const void *weights, const void *feat, const void *dir_enc, const void *app, uint32_t n_app, uint32_t S,
                     uint32_t n_seg, uint32_t act_c, const float *delta, const float *t, const uint32_t *seg_ray,
                     const uint32_t *seg_slot, uint32_t k_max, float *Ck, float *Tk, float *Dk, hipStream_t st)
{
    using namespace dg_mlp_mfma;
    const uint32_t blocks_needed = (n_seg + kWavesPerBlock - 1) / kWavesPerBlock;
    const uint32_t grid = blocks_needed < 2048 ? blocks_needed : 2048;
    const __half *w = (const __half *)weights, *f = (const __half *)feat, *dr = (const __half *)dir_enc, *ap = (const __half *)app;
    if (n_app == 0) render_fwd_kernel<0><<<grid, kBlock, 0, st>>>(w, f, dr, ap, S, n_seg, act_c, delta, t, seg_ray, seg_slot, k_max, Ck, Tk, Dk);
    else if (n_app == 16) render_fwd_kernel<16><<<grid, kBlock, 0, st>>>(w, f, dr, ap, S, n_seg, act_c, delta, t, seg_ray, seg_slot, k_max, Ck, Tk, Dk);
    else render_fwd_kernel<48><<<grid, kBlock, 0, st>>>(w, f, dr, ap, S, n_seg, act_c, delta, t, seg_ray, seg_slot, k_max, Ck, Tk, Dk);
}

void mlp_mfma_bwd(const void *weights, const void *feat, const void *dir_enc, const void *app, uint32_t n_app, uint32_t S,
                  uint64_t N, uint32_t act_c, const float *dsigma, const float *drgb, float loss_scale, float *dfeat, float *dW,
                  void *ws, hipStream_t st)
{
    using namespace dg_mlp_mfma;
    const uint64_t tiles = (N + 31) / 32, blocks_needed = (tiles + kWavesPerBlock - 1) / kWavesPerBlock;
    const uint32_t grid_c = (uint32_t)(blocks_needed < kGridColour ? blocks_needed : kGridColour);
    const uint32_t grid_d = (uint32_t)(blocks_needed < kGridDensity ? blocks_needed : kGridDensity);
    char *base = static_cast<char *>(ws);
    float *density_shares = reinterpret_cast<float *>(base);
    float *colour_shares = reinterpret_cast<float *>(base + align256((size_t)kGridDensity * kWavesPerBlock * oWc1 * sizeof(float)));
    h8 *dgeo = reinterpret_cast<h8 *>(reinterpret_cast<char *>(colour_shares) +
                                      align256((size_t)kGridColour * kWavesPerBlock * (kTotal - oWc1) * sizeof(float)));
    float *row_delta = reinterpret_cast<float *>(reinterpret_cast<char *>(dgeo) + align256((size_t)N * 32));
    const uint64_t n_rows = n_app ? (N + S - 1) / S : 0;
    const __half *w = (const __half *)weights, *f = (const __half *)feat, *dr = (const __half *)dir_enc, *ap = (const __half *)app;
    if (n_app) {
        const uint64_t n = n_rows * HC, want = (n + kBlock - 1) / kBlock;
        zero_kernel<<<(uint32_t)(want < 4096 ? want : 4096), kBlock, 0, st>>>(row_delta, n);
    }
    if (n_app == 0)
        colour_bwd_kernel<0><<<grid_c, kBlock, 0, st>>>(w, f, dr, ap, S, N, act_c, dsigma, drgb, loss_scale, dgeo, colour_shares, row_delta);
    else if (n_app == 16)
        colour_bwd_kernel<16><<<grid_c, kBlock, 0, st>>>(w, f, dr, ap, S, N, act_c, dsigma, drgb, loss_scale, dgeo, colour_shares, row_delta);
    else
        colour_bwd_kernel<48><<<grid_c, kBlock, 0, st>>>(w, f, dr, ap, S, N, act_c, dsigma, drgb, loss_scale, dgeo, colour_shares, row_delta);
    density_bwd_kernel<<<grid_d, kBlock, 0, st>>>(w, f, N, dgeo, loss_scale, dfeat, density_shares);
    fold_shares_kernel<<<(kTotal + kFoldElems - 1) / kFoldElems, kFoldElems * kFoldGroups, 0, st>>>(
        density_shares, grid_d * kWavesPerBlock, colour_shares, grid_c * kWavesPerBlock, 1.0f / loss_scale, dW);
    if (n_app) {
        const uint64_t batches = (n_rows + 8 * kWgradGroups - 1) / (8 * kWgradGroups);
        const uint32_t grid_a = (uint32_t)(batches < kWgradGrid ? batches : kWgradGrid);
        if (n_app == 16) appearance_wgrad_kernel<16><<<grid_a, kWgradBlock, 0, st>>>(row_delta, ap, n_rows, 1.0f / loss_scale, dW);
        else appearance_wgrad_kernel<48><<<grid_a, kWgradBlock, 0, st>>>(row_delta, ap, n_rows, 1.0f / loss_scale, dW);
    }
}

}  // namespace dg
