// Local volume rendering of segments, segmented merge and loss seeds (Eq. 3, Eq. 5-10).
//
// Compositing: a group of G lanes per segment, one sample per lane (G = 64, a whole wavefront, for the fixed sample
// counts: S = 64 fills it exactly; other S run in chunks of G with a carried transmittance), so sigma / rgb / delta
// are read coalesced and the front-to-back product becomes a prefix scan over the group.  Segments of different
// lengths (occupancy-guided sampling keeps 7 samples per segment on average) take G = 16: four segments per wavefront.
#include "dg_internal.h"

namespace {

constexpr int kBlock = 256;
constexpr int kWavesPerBlock = kBlock / dg::kWave;
constexpr int kRaggedGroup = 16;                   // lanes per segment where segments differ in length
constexpr int kRaggedPerBlock = kBlock / kRaggedGroup;

template <int G>
__device__ __forceinline__ float group_inclusive_product(float v, int lane)
{
#pragma unroll
    for (int off = 1; off < G; off <<= 1) {
        const float up = __shfl_up(v, off, G);
        if (lane >= off) v *= up;
    }
    return v;
}

template <int G>
__device__ __forceinline__ float group_inclusive_sum(float v, int lane)
{
#pragma unroll
    for (int off = 1; off < G; off <<= 1) {
        const float up = __shfl_up(v, off, G);
        if (lane >= off) v += up;
    }
    return v;
}

template <int G>
__device__ __forceinline__ float group_sum(float v)
{
#pragma unroll
    for (int off = G / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, G);
    return v;
}

// Every exchange below stays inside a group, and the lanes of a group run the same loops and branches (they depend on
// the segment alone), so a lane never reads from one that is switched off.
template <int G>
__global__ void __launch_bounds__(kBlock)
composite_fwd_kernel(const float *__restrict__ sigma, const float *__restrict__ rgb, const float *__restrict__ delta,
                     uint32_t n_seg, uint32_t S_fixed, const uint32_t *__restrict__ first, const uint32_t *__restrict__ seg_ray,
                     const uint32_t *__restrict__ seg_slot, uint32_t k_max, float *__restrict__ Ck,
                     float *__restrict__ Tk)
{
    const uint32_t j = blockIdx.x * (kBlock / G) + threadIdx.x / G;
    const int lane = threadIdx.x % G;
    if (j >= n_seg) return;
    const size_t begin = first ? (size_t)first[j] : (size_t)j * S_fixed;      // segments of different lengths bring their offsets
    const uint32_t S = first ? first[j + 1] - first[j] : S_fixed;
    float trans = 1.0f, c0 = 0.0f, c1 = 0.0f, c2 = 0.0f;
    for (uint32_t base = 0; base < S; base += G) {
        const uint32_t s = base + lane;
        const bool live = s < S;
        const size_t n = begin + (live ? s : 0);
        const float x = live ? sigma[n] * delta[n] : 0.0f;
        const float keep = expf(-x);                        // 1 - alpha
        const float alpha = -expm1f(-x);
        const float incl = group_inclusive_product<G>(keep, lane);
        float before = __shfl_up(incl, 1, G);
        if (lane == 0) before = 1.0f;
        const float wgt = live ? trans * before * alpha : 0.0f;
        c0 += wgt * (live ? rgb[3 * n] : 0.0f);
        c1 += wgt * (live ? rgb[3 * n + 1] : 0.0f);
        c2 += wgt * (live ? rgb[3 * n + 2] : 0.0f);
        trans *= __shfl(incl, G - 1, G);
    }
    c0 = group_sum<G>(c0); c1 = group_sum<G>(c1); c2 = group_sum<G>(c2);
    if (lane == 0) {
        const size_t dst = (size_t)seg_ray[j] * k_max + seg_slot[j];
        Ck[3 * dst] = c0; Ck[3 * dst + 1] = c1; Ck[3 * dst + 2] = c2;
        Tk[dst] = trans;
    }
}

// Depth of evaluation rendering (Sec. 4.4.2): D_k = sum_i T_i alpha_i t_i, the colour rule applied to the sample distances
template <int G>
__global__ void __launch_bounds__(kBlock)
composite_depth_kernel(const float *__restrict__ sigma, const float *__restrict__ delta, const float *__restrict__ t,
                       uint32_t n_seg, uint32_t S_fixed, const uint32_t *__restrict__ first, const uint32_t *__restrict__ seg_ray,
                       const uint32_t *__restrict__ seg_slot, uint32_t k_max, float *__restrict__ Dk)
{
    const uint32_t j = blockIdx.x * (kBlock / G) + threadIdx.x / G;
    const int lane = threadIdx.x % G;
    if (j >= n_seg) return;
    const size_t begin = first ? (size_t)first[j] : (size_t)j * S_fixed;      // segments of different lengths bring their offsets
    const uint32_t S = first ? first[j + 1] - first[j] : S_fixed;
    float trans = 1.0f, depth = 0.0f;
    for (uint32_t base = 0; base < S; base += G) {
        const uint32_t s = base + lane;
        const bool live = s < S;
        const size_t n = begin + (live ? s : 0);
        const float x = live ? sigma[n] * delta[n] : 0.0f;
        const float incl = group_inclusive_product<G>(expf(-x), lane);
        float before = __shfl_up(incl, 1, G);
        if (lane == 0) before = 1.0f;
        depth += live ? trans * before * -expm1f(-x) * t[n] : 0.0f;
        trans *= __shfl(incl, G - 1, G);
    }
    depth = group_sum<G>(depth);
    if (lane == 0) Dk[(size_t)seg_ray[j] * k_max + seg_slot[j]] = depth;
}

// d sigma_i = delta_i [ gC.(T_{i+1} c_i) - sum_{j>i} w_j gC.c_j - gT T_k ],  d c_i = w_i gC
template <int G>
__global__ void __launch_bounds__(kBlock)
composite_bwd_kernel(const float *__restrict__ sigma, const float *__restrict__ rgb, const float *__restrict__ delta,
                     uint32_t n_seg, uint32_t S_fixed, const uint32_t *__restrict__ first, const uint32_t *__restrict__ seg_ray,
                     const uint32_t *__restrict__ seg_slot, uint32_t k_max, const float *__restrict__ gCk,
                     const float *__restrict__ gTk, float *__restrict__ dsigma, float *__restrict__ drgb)
{
    const uint32_t j = blockIdx.x * (kBlock / G) + threadIdx.x / G;
    const int lane = threadIdx.x % G;
    if (j >= n_seg) return;
    const size_t begin = first ? (size_t)first[j] : (size_t)j * S_fixed;      // segments of different lengths bring their offsets
    const uint32_t S = first ? first[j + 1] - first[j] : S_fixed;
    const size_t src = (size_t)seg_ray[j] * k_max + seg_slot[j];
    const float g0 = gCk[3 * src], g1 = gCk[3 * src + 1], g2 = gCk[3 * src + 2], gt = gTk[src];

    // pass 1 (only needed when the segment spans several chunks): total of q_j = w_j gC.c_j and T_k
    float total_q = 0.0f, trans_all = 1.0f;
    if (S > (uint32_t)G) {
        float trans = 1.0f, q = 0.0f;
        for (uint32_t base = 0; base < S; base += G) {
            const uint32_t s = base + lane;
            const bool live = s < S;
            const size_t n = begin + (live ? s : 0);
            const float x = live ? sigma[n] * delta[n] : 0.0f;
            const float incl = group_inclusive_product<G>(expf(-x), lane);
            float before = __shfl_up(incl, 1, G);
            if (lane == 0) before = 1.0f;
            const float wgt = live ? trans * before * -expm1f(-x) : 0.0f;
            if (live) q += wgt * (g0 * rgb[3 * n] + g1 * rgb[3 * n + 1] + g2 * rgb[3 * n + 2]);
            trans *= __shfl(incl, G - 1, G);
        }
        total_q = group_sum<G>(q);
        trans_all = trans;
    }

    float trans = 1.0f, q_before = 0.0f;      // running transmittance and running sum of q over earlier chunks
    for (uint32_t base = 0; base < S; base += G) {
        const uint32_t s = base + lane;
        const bool live = s < S;
        const size_t n = begin + (live ? s : 0);
        const float dl = live ? delta[n] : 0.0f;
        const float x = live ? sigma[n] * dl : 0.0f;
        const float keep = expf(-x);
        const float incl = group_inclusive_product<G>(keep, lane);
        float before = __shfl_up(incl, 1, G);
        if (lane == 0) before = 1.0f;
        const float t_before = trans * before;
        const float wgt = live ? t_before * -expm1f(-x) : 0.0f;
        const float r0 = live ? rgb[3 * n] : 0.0f, r1 = live ? rgb[3 * n + 1] : 0.0f, r2 = live ? rgb[3 * n + 2] : 0.0f;
        const float gc = g0 * r0 + g1 * r1 + g2 * r2;
        const float q = wgt * gc;
        const float q_incl = group_inclusive_sum<G>(q, lane);
        const float chunk_q = __shfl(q_incl, G - 1, G);
        const float chunk_keep = __shfl(incl, G - 1, G);
        if (S <= (uint32_t)G) { total_q = chunk_q; trans_all = chunk_keep; }
        const float behind = total_q - (q_before + q_incl);
        if (live) {
            dsigma[n] = dl * (t_before * keep * gc - behind - gt * trans_all);
            drgb[3 * n] = wgt * g0; drgb[3 * n + 1] = wgt * g1; drgb[3 * n + 2] = wgt * g2;
        }
        q_before += chunk_q;
        trans *= chunk_keep;
    }
}

constexpr uint32_t kMaxK = 12;

__global__ void __launch_bounds__(kBlock)
merge_fwd_kernel(const float *__restrict__ Ck, const float *__restrict__ Tk, const uint32_t *__restrict__ seg_count,
                 uint32_t R, uint32_t k_max, float *__restrict__ C, float *__restrict__ T)
{
    const uint32_t r = blockIdx.x * kBlock + threadIdx.x;
    if (r >= R) return;
    const uint32_t K = min(seg_count[r], k_max);
    float front = 1.0f, c0 = 0.0f, c1 = 0.0f, c2 = 0.0f;
    for (uint32_t k = 0; k < K; ++k) {
        const size_t i = (size_t)r * k_max + k;
        c0 += front * Ck[3 * i]; c1 += front * Ck[3 * i + 1]; c2 += front * Ck[3 * i + 2];
        front *= Tk[i];
    }
    C[3 * r] = c0; C[3 * r + 1] = c1; C[3 * r + 2] = c2;
    T[r] = front;
}

// depth merges like a colour channel under Eq. 5
__global__ void __launch_bounds__(kBlock)
merge_depth_kernel(const float *__restrict__ Dk, const float *__restrict__ Tk, const uint32_t *__restrict__ seg_count,
                   uint32_t R, uint32_t k_max, float *__restrict__ D)
{
    const uint32_t r = blockIdx.x * kBlock + threadIdx.x;
    if (r >= R) return;
    const uint32_t K = min(seg_count[r], k_max);
    float front = 1.0f, depth = 0.0f;
    for (uint32_t k = 0; k < K; ++k) {
        const size_t i = (size_t)r * k_max + k;
        depth += front * Dk[i];
        front *= Tk[i];
    }
    D[r] = depth;
}

// Eq. 7: gC_k = gC P_k with P_k = prod_{j<k} T_j.
// Eq. 8 regrouped so that no T_k is divided out: with the suffix values
//   A_k = sum_{m>k} (prod_{k<j<m} T_j) gC.C_m   and   B_k = prod_{j>k} T_j,
// gT_k = P_k (gT B_k + A_k); A and B follow from a back-to-front sweep.
__global__ void __launch_bounds__(kBlock)
merge_bwd_kernel(const float *__restrict__ Ck, const float *__restrict__ Tk, const uint32_t *__restrict__ seg_count,
                 uint32_t R, uint32_t k_max, const float *__restrict__ gC, const float *__restrict__ gT,
                 float *__restrict__ gCk, float *__restrict__ gTk)
{
    const uint32_t r = blockIdx.x * kBlock + threadIdx.x;
    if (r >= R) return;
    const uint32_t K = min(seg_count[r], k_max);
    const float g0 = gC[3 * r], g1 = gC[3 * r + 1], g2 = gC[3 * r + 2], gt = gT[r];
    float tk[kMaxK], front[kMaxK];
    float p = 1.0f;
    for (uint32_t k = 0; k < kMaxK; ++k) {
        if (k < K) { tk[k] = Tk[(size_t)r * k_max + k]; front[k] = p; p *= tk[k]; }
    }
    float a = 0.0f, b = 1.0f;
    for (int k = (int)kMaxK - 1; k >= 0; --k) {
        const size_t i = (size_t)r * k_max + k;
        if ((uint32_t)k < K) {
            gTk[i] = front[k] * (gt * b + a);
            gCk[3 * i] = g0 * front[k]; gCk[3 * i + 1] = g1 * front[k]; gCk[3 * i + 2] = g2 * front[k];
            const float gc = g0 * Ck[3 * i] + g1 * Ck[3 * i + 1] + g2 * Ck[3 * i + 2];
            a = gc + tk[k] * a;
            b *= tk[k];
        } else if ((uint32_t)k < k_max) {
            gTk[i] = 0.0f; gCk[3 * i] = 0.0f; gCk[3 * i + 1] = 0.0f; gCk[3 * i + 2] = 0.0f;
        }
    }
}

__global__ void __launch_bounds__(kBlock)
loss_seed_kernel(const float *__restrict__ C, const float *__restrict__ T, const float *__restrict__ Cgt, uint32_t R,
                 float lambda1, float *__restrict__ gC, float *__restrict__ gT, float *__restrict__ loss)
{
    __shared__ float partial[kWavesPerBlock];
    const uint32_t r = blockIdx.x * kBlock + threadIdx.x;
    const float inv_r = 1.0f / (float)R;
    float mine = 0.0f;
    if (r < R) {
        for (int c = 0; c < 3; ++c) {
            const float e = C[3 * r + c] - Cgt[3 * r + c];
            mine += e * e * inv_r;
            gC[3 * r + c] = 2.0f * e * inv_r;
        }
        const float opaque = 1.0f - T[r];
        const bool clamped = !(opaque >= 1e-6f);
        gT[r] = clamped ? 0.0f : lambda1 * inv_r / opaque;
        if (lambda1 != 0.0f) mine -= lambda1 * inv_r * logf(clamped ? 1e-6f : opaque);
    }
    if (loss) {
        mine = group_sum<dg::kWave>(mine);
        if (threadIdx.x % dg::kWave == 0) partial[threadIdx.x / dg::kWave] = mine;
        __syncthreads();
        if (threadIdx.x == 0) {
            float s = 0.0f;
            for (int w = 0; w < kWavesPerBlock; ++w) s += partial[w];
            atomicAdd(loss, s);
        }
    }
}

int seg_args_ok(uint32_t n_seg, uint32_t S, uint32_t k_max, const char *who)
{
    DG_REQUIRE(S >= 1 && k_max >= 1, DG_ERR_ARG, "%s: S and k_max must be >= 1", who);
    DG_REQUIRE((uint64_t)n_seg + kWavesPerBlock - 1 <= 0x7fffffffull * kWavesPerBlock, DG_ERR_UNSUPPORTED, "%s: too many segments", who);
    return DG_OK;
}

}  // namespace

extern "C" int dg_composite_segment_fwd(const float *sigma, const float *rgb, const float *delta, uint32_t n_seg,
                                        uint32_t S, const uint32_t *seg_ray, const uint32_t *seg_slot, uint32_t k_max,
                                        float *Ck, float *Tk, void *stream)
{
    if (int rc = seg_args_ok(n_seg, S, k_max, "dg_composite_segment_fwd")) return rc;
    if (n_seg == 0) return DG_OK;
    DG_REQUIRE(sigma && rgb && delta && seg_ray && seg_slot && Ck && Tk, DG_ERR_ARG, "dg_composite_segment_fwd: null pointer");
    const uint32_t n_blocks = (n_seg + kWavesPerBlock - 1) / kWavesPerBlock;
    composite_fwd_kernel<dg::kWave><<<n_blocks, kBlock, 0, (hipStream_t)stream>>>(sigma, rgb, delta, n_seg, S, nullptr, seg_ray,
                                                                       seg_slot, k_max, Ck, Tk);
    return dg::launch_status("dg_composite_segment_fwd");
}

extern "C" int dg_composite_segment_depth(const float *sigma, const float *delta, const float *t, uint32_t n_seg, uint32_t S,
                                          const uint32_t *seg_ray, const uint32_t *seg_slot, uint32_t k_max, float *Dk,
                                          void *stream)
{
    if (int rc = seg_args_ok(n_seg, S, k_max, "dg_composite_segment_depth")) return rc;
    if (n_seg == 0) return DG_OK;
    DG_REQUIRE(sigma && delta && t && seg_ray && seg_slot && Dk, DG_ERR_ARG, "dg_composite_segment_depth: null pointer");
    const uint32_t n_blocks = (n_seg + kWavesPerBlock - 1) / kWavesPerBlock;
    composite_depth_kernel<dg::kWave><<<n_blocks, kBlock, 0, (hipStream_t)stream>>>(sigma, delta, t, n_seg, S, nullptr, seg_ray, seg_slot,
                                                                         k_max, Dk);
    return dg::launch_status("dg_composite_segment_depth");
}

extern "C" int dg_composite_segment_bwd(const float *sigma, const float *rgb, const float *delta, uint32_t n_seg,
                                        uint32_t S, const uint32_t *seg_ray, const uint32_t *seg_slot, uint32_t k_max,
                                        const float *gCk, const float *gTk, float *dsigma, float *drgb, void *stream)
{
    if (int rc = seg_args_ok(n_seg, S, k_max, "dg_composite_segment_bwd")) return rc;
    if (n_seg == 0) return DG_OK;
    DG_REQUIRE(sigma && rgb && delta && seg_ray && seg_slot && gCk && gTk && dsigma && drgb, DG_ERR_ARG,
               "dg_composite_segment_bwd: null pointer");
    const uint32_t n_blocks = (n_seg + kWavesPerBlock - 1) / kWavesPerBlock;
    composite_bwd_kernel<dg::kWave><<<n_blocks, kBlock, 0, (hipStream_t)stream>>>(sigma, rgb, delta, n_seg, S, nullptr, seg_ray,
                                                                       seg_slot, k_max, gCk, gTk, dsigma, drgb);
    return dg::launch_status("dg_composite_segment_bwd");
}

// ---- the same three on segments of different lengths (occupancy-guided sampling, Sec. 3.2 / Sec. 5.1)
extern "C" int dg_composite_ragged_fwd(const float *sigma, const float *rgb, const float *delta, uint32_t n_seg,
                                       const uint32_t *first, const uint32_t *seg_ray, const uint32_t *seg_slot, uint32_t k_max,
                                       float *Ck, float *Tk, void *stream)
{
    if (int rc = seg_args_ok(n_seg, 1, k_max, "dg_composite_ragged_fwd")) return rc;
    if (n_seg == 0) return DG_OK;
    DG_REQUIRE(sigma && rgb && delta && first && seg_ray && seg_slot && Ck && Tk, DG_ERR_ARG, "dg_composite_ragged_fwd: null pointer");
    const uint32_t n_blocks = (n_seg + kRaggedPerBlock - 1) / kRaggedPerBlock;
    composite_fwd_kernel<kRaggedGroup><<<n_blocks, kBlock, 0, (hipStream_t)stream>>>(sigma, rgb, delta, n_seg, 0, first, seg_ray, seg_slot,
                                                                       k_max, Ck, Tk);
    return dg::launch_status("dg_composite_ragged_fwd");
}

extern "C" int dg_composite_ragged_depth(const float *sigma, const float *delta, const float *t, uint32_t n_seg,
                                         const uint32_t *first, const uint32_t *seg_ray, const uint32_t *seg_slot, uint32_t k_max,
                                         float *Dk, void *stream)
{
    if (int rc = seg_args_ok(n_seg, 1, k_max, "dg_composite_ragged_depth")) return rc;
    if (n_seg == 0) return DG_OK;
    DG_REQUIRE(sigma && delta && t && first && seg_ray && seg_slot && Dk, DG_ERR_ARG, "dg_composite_ragged_depth: null pointer");
    const uint32_t n_blocks = (n_seg + kRaggedPerBlock - 1) / kRaggedPerBlock;
    composite_depth_kernel<kRaggedGroup><<<n_blocks, kBlock, 0, (hipStream_t)stream>>>(sigma, delta, t, n_seg, 0, first, seg_ray, seg_slot,
                                                                         k_max, Dk);
    return dg::launch_status("dg_composite_ragged_depth");
}

extern "C" int dg_composite_ragged_bwd(const float *sigma, const float *rgb, const float *delta, uint32_t n_seg,
                                       const uint32_t *first, const uint32_t *seg_ray, const uint32_t *seg_slot, uint32_t k_max,
                                       const float *gCk, const float *gTk, float *dsigma, float *drgb, void *stream)
{
    if (int rc = seg_args_ok(n_seg, 1, k_max, "dg_composite_ragged_bwd")) return rc;
    if (n_seg == 0) return DG_OK;
    DG_REQUIRE(sigma && rgb && delta && first && seg_ray && seg_slot && gCk && gTk && dsigma && drgb, DG_ERR_ARG,
               "dg_composite_ragged_bwd: null pointer");
    const uint32_t n_blocks = (n_seg + kRaggedPerBlock - 1) / kRaggedPerBlock;
    composite_bwd_kernel<kRaggedGroup><<<n_blocks, kBlock, 0, (hipStream_t)stream>>>(sigma, rgb, delta, n_seg, 0, first, seg_ray, seg_slot,
                                                                       k_max, gCk, gTk, dsigma, drgb);
    return dg::launch_status("dg_composite_ragged_bwd");
}

extern "C" int dg_merge_segments(const float *Ck, const float *Tk, const uint32_t *seg_count, uint32_t R,
                                 uint32_t k_max, float *C, float *T, void *stream)
{
    DG_REQUIRE(k_max >= 1 && k_max <= kMaxK, DG_ERR_UNSUPPORTED, "dg_merge_segments: k_max=%u outside 1..%u", k_max, kMaxK);
    if (R == 0) return DG_OK;
    DG_REQUIRE(Ck && Tk && seg_count && C && T, DG_ERR_ARG, "dg_merge_segments: null pointer");
    merge_fwd_kernel<<<(R + kBlock - 1) / kBlock, kBlock, 0, (hipStream_t)stream>>>(Ck, Tk, seg_count, R, k_max, C, T);
    return dg::launch_status("dg_merge_segments");
}

extern "C" int dg_merge_depth(const float *Dk, const float *Tk, const uint32_t *seg_count, uint32_t R, uint32_t k_max,
                              float *D, void *stream)
{
    DG_REQUIRE(k_max >= 1 && k_max <= kMaxK, DG_ERR_UNSUPPORTED, "dg_merge_depth: k_max=%u outside 1..%u", k_max, kMaxK);
    if (R == 0) return DG_OK;
    DG_REQUIRE(Dk && Tk && seg_count && D, DG_ERR_ARG, "dg_merge_depth: null pointer");
    merge_depth_kernel<<<(R + kBlock - 1) / kBlock, kBlock, 0, (hipStream_t)stream>>>(Dk, Tk, seg_count, R, k_max, D);
    return dg::launch_status("dg_merge_depth");
}

extern "C" int dg_merge_segments_bwd(const float *Ck, const float *Tk, const uint32_t *seg_count, uint32_t R,
                                     uint32_t k_max, const float *gC, const float *gT, float *gCk, float *gTk,
                                     void *stream)
{
    DG_REQUIRE(k_max >= 1 && k_max <= kMaxK, DG_ERR_UNSUPPORTED, "dg_merge_segments_bwd: k_max=%u outside 1..%u", k_max, kMaxK);
    if (R == 0) return DG_OK;
    DG_REQUIRE(Ck && Tk && seg_count && gC && gT && gCk && gTk, DG_ERR_ARG, "dg_merge_segments_bwd: null pointer");
    merge_bwd_kernel<<<(R + kBlock - 1) / kBlock, kBlock, 0, (hipStream_t)stream>>>(Ck, Tk, seg_count, R, k_max, gC, gT,
                                                                                    gCk, gTk);
    return dg::launch_status("dg_merge_segments_bwd");
}

extern "C" int dg_loss_seed(const float *C, const float *T, const float *Cgt, uint32_t R, float lambda1, float *gC,
                            float *gT, float *loss, void *stream)
{
    if (R == 0) return DG_OK;
    DG_REQUIRE(C && T && Cgt && gC && gT, DG_ERR_ARG, "dg_loss_seed: null pointer");
    loss_seed_kernel<<<(R + kBlock - 1) / kBlock, kBlock, 0, (hipStream_t)stream>>>(C, T, Cgt, R, lambda1, gC, gT, loss);
    return dg::launch_status("dg_loss_seed");
}
