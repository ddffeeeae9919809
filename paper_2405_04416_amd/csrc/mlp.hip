// Field MLPs: density net then colour net (Sec. 3.2; activations and output clip of Sec. 5.1).
//
// Reference-shaped kernels: one sample per lane, weights broadcast from LDS, fp16 rounding at the
// documented points, fp32 accumulation.  The backward recomputes the forward, stages each layer's
// (delta, activation) pair in LDS and lets every thread own a slice of dW, accumulated in registers
// across the tiles a persistent workgroup visits; per-workgroup partial sums go to the workspace and
// a second kernel folds them into dW in a fixed order.
#include "dg_internal.h"

namespace {

template <int NF, int HD, int NG, int ND, int HC, int NLC>
struct Net {
    static constexpr int kNF = NF, kHD = HD, kNG = NG, kND = ND, kHC = HC, kNLC = NLC, kCI = NG + ND;
    static constexpr int oWd1 = 0;
    static constexpr int oWd2 = oWd1 + HD * NF;
    static constexpr int oWc1 = oWd2 + NG * HD;
    static constexpr int oWc2 = oWc1 + HC * (NG + ND);
    static constexpr int oWc3 = oWc2 + (NLC == 2 ? HC * HC : 0);
    static constexpr int kTotal = oWc3 + 3 * HC;
};

__device__ __forceinline__ float r16(float x) { return __half2float(__float2half_rn(x)); }
__device__ __forceinline__ float clip15(float x) { return fminf(fmaxf(x, -15.0f), 15.0f); }
__device__ __forceinline__ float sigmoidf(float x) { return 1.0f / (1.0f + expf(-x)); }
__device__ __forceinline__ float act(uint32_t kind, float x) { return kind ? sigmoidf(x) : fmaxf(x, 0.0f); }
__device__ __forceinline__ float dact(uint32_t kind, float a) { return kind ? a * (1.0f - a) : (a > 0.0f ? 1.0f : 0.0f); }

template <int NOUT, int NIN>
__device__ __forceinline__ void matvec(const __half *W, const float *x, float *y)
{
    for (int o = 0; o < NOUT; ++o) {
        float s = 0.0f;
#pragma unroll 8
        for (int i = 0; i < NIN; ++i) s = fmaf(__half2float(W[o * NIN + i]), x[i], s);
        y[o] = s;
    }
}

template <int NOUT, int NIN>
__device__ __forceinline__ void matvec_t(const __half *W, const float *y, float *x, int n_in_used = NIN)
{
    for (int i = 0; i < n_in_used; ++i) {
        float s = 0.0f;
#pragma unroll 8
        for (int o = 0; o < NOUT; ++o) s = fmaf(__half2float(W[o * NIN + i]), y[o], s);
        x[i] = s;
    }
}

template <class N>
struct Acts {
    float x0[N::kNF], h1[N::kHD], geo[N::kNG], xc[N::kCI], c1[N::kHC], c2[N::kNLC == 2 ? N::kHC : 1], raw[3];
    float sigma, rgb[3];
};

template <class N>
__device__ __forceinline__ void forward_one(const __half *w, const __half *feat, uint64_t n_samples, uint64_t n,
                                            const __half *dir_row, uint32_t act_c, Acts<N> &a)
{
    float z[N::kHD > N::kHC ? N::kHD : N::kHC];
    // features are level-major planes [n_feat / 2][n_samples][2]
    for (int i = 0; i < N::kNF; ++i) a.x0[i] = __half2float(feat[((size_t)(i >> 1) * n_samples + n) * 2 + (i & 1)]);
    matvec<N::kHD, N::kNF>(w + N::oWd1, a.x0, z);
    for (int i = 0; i < N::kHD; ++i) a.h1[i] = r16(fmaxf(z[i], 0.0f));
    matvec<N::kNG, N::kHD>(w + N::oWd2, a.h1, a.geo);
    a.sigma = expf(clip15(a.geo[0]));
    for (int i = 0; i < N::kNG; ++i) a.xc[i] = r16(a.geo[i]);
    for (int i = 0; i < N::kND; ++i) a.xc[N::kNG + i] = __half2float(dir_row[i]);
    matvec<N::kHC, N::kCI>(w + N::oWc1, a.xc, z);
    for (int i = 0; i < N::kHC; ++i) a.c1[i] = r16(act(act_c, z[i]));
    const float *last = a.c1;
    if (N::kNLC == 2) {
        matvec<N::kHC, N::kHC>(w + N::oWc2, a.c1, z);
        for (int i = 0; i < N::kHC; ++i) a.c2[i] = r16(act(act_c, z[i]));
        last = a.c2;
    }
    matvec<3, N::kHC>(w + N::oWc3, last, a.raw);
    for (int c = 0; c < 3; ++c) a.rgb[c] = sigmoidf(clip15(a.raw[c]));
}

constexpr int kFwdBlock = 128;

template <class N>
__global__ void __launch_bounds__(kFwdBlock)
mlp_fwd_kernel(const __half *__restrict__ weights, const __half *__restrict__ feat, const __half *__restrict__ dir_enc,
               uint32_t S, uint64_t n_samples, uint32_t act_c, float *__restrict__ sigma, float *__restrict__ rgb)
{
    __shared__ __half w[N::kTotal];
    for (int i = threadIdx.x; i < N::kTotal; i += kFwdBlock) w[i] = weights[i];
    __syncthreads();
    const uint64_t n = (uint64_t)blockIdx.x * kFwdBlock + threadIdx.x;
    if (n >= n_samples) return;
    Acts<N> a;
    forward_one<N>(w, feat, n_samples, n, dir_enc + (n / S) * N::kND, act_c, a);
    sigma[n] = a.sigma;
    rgb[3 * n] = a.rgb[0]; rgb[3 * n + 1] = a.rgb[1]; rgb[3 * n + 2] = a.rgb[2];
}

constexpr int kBwdBlock = 128;

// dW slice owned by one thread: entries e = tid, tid + kBwdBlock, ... of a [NOUT, NIN] block
template <int NOUT, int NIN>
__device__ __forceinline__ void wgrad_tile(const __half *dl, const __half *av, int n_live, float *acc)
{
    constexpr int kPer = (NOUT * NIN + kBwdBlock - 1) / kBwdBlock;
#pragma unroll
    for (int q = 0; q < kPer; ++q) {
        const int e = threadIdx.x + q * kBwdBlock;
        if (e < NOUT * NIN) {
            const int o = e / NIN, i = e % NIN;
            float s = 0.0f;
            for (int t = 0; t < n_live; ++t) s = fmaf(__half2float(dl[t * NOUT + o]), __half2float(av[t * NIN + i]), s);
            acc[q] += s;
        }
    }
}

template <int NOUT, int NIN>
__device__ __forceinline__ void stage(__half *dl, __half *av, const float *delta, const float *activ, bool live)
{
    __syncthreads();      // previous layer's readers are done
    for (int o = 0; o < NOUT; ++o) dl[threadIdx.x * NOUT + o] = __float2half_rn(live ? delta[o] : 0.0f);
    for (int i = 0; i < NIN; ++i) av[threadIdx.x * NIN + i] = __float2half_rn(live ? activ[i] : 0.0f);
    __syncthreads();
}

template <int NOUT, int NIN>
__device__ __forceinline__ void flush(const float *acc, float *dst)
{
    constexpr int kPer = (NOUT * NIN + kBwdBlock - 1) / kBwdBlock;
#pragma unroll
    for (int q = 0; q < kPer; ++q) {
        const int e = threadIdx.x + q * kBwdBlock;
        if (e < NOUT * NIN) dst[e] = acc[q];
    }
}

template <class N>
__global__ void __launch_bounds__(kBwdBlock)
mlp_bwd_kernel(const __half *__restrict__ weights, const __half *__restrict__ feat, const __half *__restrict__ dir_enc,
               uint32_t S, uint64_t n_samples, uint32_t act_c, const float *__restrict__ dsigma,
               const float *__restrict__ drgb, float loss_scale, float *__restrict__ dfeat,
               float *__restrict__ partial)
{
    constexpr int kMaxOut = N::kHD > N::kHC ? N::kHD : N::kHC;
    constexpr int kMaxIn = kMaxOut > N::kCI ? (kMaxOut > N::kNF ? kMaxOut : N::kNF) : (N::kCI > N::kNF ? N::kCI : N::kNF);
    __shared__ __half w[N::kTotal];
    __shared__ __half s_dl[kBwdBlock * kMaxOut];
    __shared__ __half s_av[kBwdBlock * kMaxIn];
    for (int i = threadIdx.x; i < N::kTotal; i += kBwdBlock) w[i] = weights[i];
    __syncthreads();

    constexpr int pWd1 = (N::kHD * N::kNF + kBwdBlock - 1) / kBwdBlock;
    constexpr int pWd2 = (N::kNG * N::kHD + kBwdBlock - 1) / kBwdBlock;
    constexpr int pWc1 = (N::kHC * N::kCI + kBwdBlock - 1) / kBwdBlock;
    constexpr int pWc2 = N::kNLC == 2 ? (N::kHC * N::kHC + kBwdBlock - 1) / kBwdBlock : 1;
    constexpr int pWc3 = (3 * N::kHC + kBwdBlock - 1) / kBwdBlock;
    float aWd1[pWd1] = {}, aWd2[pWd2] = {}, aWc1[pWc1] = {}, aWc2[pWc2] = {}, aWc3[pWc3] = {};

    const uint64_t n_tiles = (n_samples + kBwdBlock - 1) / kBwdBlock;
    const float inv_scale = 1.0f / loss_scale;
    for (uint64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const uint64_t n = tile * kBwdBlock + threadIdx.x;
        const bool live = n < n_samples;
        const uint64_t nn = live ? n : 0;
        const int n_live = (int)min((uint64_t)kBwdBlock, n_samples - tile * kBwdBlock);
        Acts<N> a;
        forward_one<N>(w, feat, n_samples, nn, dir_enc + (nn / S) * N::kND, act_c, a);

        float d3[3], g[kMaxIn], dl[kMaxOut];
        for (int c = 0; c < 3; ++c) {
            const bool pass = a.raw[c] >= -15.0f && a.raw[c] <= 15.0f;
            d3[c] = r16(pass ? loss_scale * drgb[3 * nn + c] * a.rgb[c] * (1.0f - a.rgb[c]) : 0.0f);
        }
        const float *last = N::kNLC == 2 ? a.c2 : a.c1;
        stage<3, N::kHC>(s_dl, s_av, d3, last, live);
        wgrad_tile<3, N::kHC>(s_dl, s_av, n_live, aWc3);
        matvec_t<3, N::kHC>(w + N::oWc3, d3, g);
        if (N::kNLC == 2) {
            for (int k = 0; k < N::kHC; ++k) dl[k] = r16(g[k] * dact(act_c, a.c2[k]));
            stage<N::kHC, N::kHC>(s_dl, s_av, dl, a.c1, live);
            wgrad_tile<N::kHC, N::kHC>(s_dl, s_av, n_live, aWc2);
            matvec_t<N::kHC, N::kHC>(w + N::oWc2, dl, g);
        }
        for (int k = 0; k < N::kHC; ++k) dl[k] = r16(g[k] * dact(act_c, a.c1[k]));
        stage<N::kHC, N::kCI>(s_dl, s_av, dl, a.xc, live);
        wgrad_tile<N::kHC, N::kCI>(s_dl, s_av, n_live, aWc1);
        matvec_t<N::kHC, N::kCI>(w + N::oWc1, dl, g, N::kNG);      // direction inputs carry no gradient
        const bool pass0 = a.geo[0] >= -15.0f && a.geo[0] <= 15.0f;
        g[0] += pass0 ? loss_scale * dsigma[nn] * a.sigma : 0.0f;
        for (int k = 0; k < N::kNG; ++k) dl[k] = r16(g[k]);
        stage<N::kNG, N::kHD>(s_dl, s_av, dl, a.h1, live);
        wgrad_tile<N::kNG, N::kHD>(s_dl, s_av, n_live, aWd2);
        matvec_t<N::kNG, N::kHD>(w + N::oWd2, dl, g);
        for (int k = 0; k < N::kHD; ++k) dl[k] = r16(a.h1[k] > 0.0f ? g[k] : 0.0f);
        stage<N::kHD, N::kNF>(s_dl, s_av, dl, a.x0, live);
        wgrad_tile<N::kHD, N::kNF>(s_dl, s_av, n_live, aWd1);
        matvec_t<N::kHD, N::kNF>(w + N::oWd1, dl, g);
        if (live)
            for (int k = 0; k < N::kNF; ++k) dfeat[((size_t)(k >> 1) * n_samples + n) * 2 + (k & 1)] = g[k] * inv_scale;
    }
    float *mine = partial + (size_t)blockIdx.x * N::kTotal;
    flush<N::kHD, N::kNF>(aWd1, mine + N::oWd1);
    flush<N::kNG, N::kHD>(aWd2, mine + N::oWd2);
    flush<N::kHC, N::kCI>(aWc1, mine + N::oWc1);
    if (N::kNLC == 2) flush<N::kHC, N::kHC>(aWc2, mine + N::oWc2);
    flush<3, N::kHC>(aWc3, mine + N::oWc3);
}

__global__ void __launch_bounds__(256)
fold_partials_kernel(const float *__restrict__ partial, uint32_t n_parts, uint32_t n_weights, float inv_scale,
                     float *__restrict__ dW)
{
    const uint32_t e = blockIdx.x * 256 + threadIdx.x;
    if (e >= n_weights) return;
    float s = 0.0f;
    for (uint32_t b = 0; b < n_parts; ++b) s += partial[(size_t)b * n_weights + e];
    dW[e] += s * inv_scale;
}

using NetNgp = Net<32, 64, 16, 16, 64, 2>;
using NetTiny = Net<8, 32, 16, 4, 32, 1>;
constexpr uint32_t kBwdGrid = 1024;   // persistent workgroups of the backward pass

int which_net(const dg_mlp_desc *m, const char *who)
{
    DG_REQUIRE(m, DG_ERR_ARG, "%s: null descriptor", who);
    DG_REQUIRE(m->act_c <= 1, DG_ERR_ARG, "%s: act_c must be 0 or 1", who);
    if (m->n_feat == 32 && m->n_hidden_d == 64 && m->n_geo == 16 && m->n_dir == 16 && m->n_hidden_c == 64 && m->n_layers_c == 2 &&
        (m->n_app == 0 || m->n_app == 16 || m->n_app == 48))
        return 1;
    if (m->n_feat == 8 && m->n_hidden_d == 32 && m->n_geo == 16 && m->n_dir == 4 && m->n_hidden_c == 32 && m->n_layers_c == 1 &&
        m->n_app == 0)
        return 2;
    return dg::fail(DG_ERR_UNSUPPORTED, "%s: unsupported MLP shape (%u,%u,%u,%u,%u,%u) with %u appearance inputs", who, m->n_feat,
                    m->n_hidden_d, m->n_geo, m->n_dir, m->n_hidden_c, m->n_layers_c, m->n_app);
}

}  // namespace

extern "C" int dg_mlp_fwd(const dg_mlp_desc *desc, const void *weights, const void *feat, const void *dir_enc,
                          uint32_t S, uint64_t N, float *sigma, float *rgb, void *stream)
{
    DG_REQUIRE(!desc || desc->n_app == 0, DG_ERR_ARG, "dg_mlp_fwd: a network with appearance inputs needs dg_mlp_fwd_app");
    return dg_mlp_fwd_app(desc, weights, feat, dir_enc, nullptr, S, N, sigma, rgb, stream);
}

extern "C" int dg_mlp_fwd_app(const dg_mlp_desc *desc, const void *weights, const void *feat, const void *dir_enc,
                              const void *app, uint32_t S, uint64_t N, float *sigma, float *rgb, void *stream)
{
    const int net = which_net(desc, "dg_mlp_fwd");
    if (net < 0) return net;
    DG_REQUIRE(S >= 1, DG_ERR_ARG, "dg_mlp_fwd: S must be >= 1");
    if (N == 0) return DG_OK;
    DG_REQUIRE(weights && feat && dir_enc && sigma && rgb, DG_ERR_ARG, "dg_mlp_fwd: null pointer");
    DG_REQUIRE(desc->n_app == 0 || (app && dg::aligned(app, 16)), DG_ERR_ARG, "dg_mlp_fwd: appearance rows missing or not 16-byte aligned");
    const uint64_t n_blocks = (N + kFwdBlock - 1) / kFwdBlock;
    DG_REQUIRE(n_blocks <= 0x7fffffffull, DG_ERR_UNSUPPORTED, "dg_mlp_fwd: N too large");
    hipStream_t st = (hipStream_t)stream;
    if (net == 1) {
        DG_REQUIRE(dg::aligned(feat, 4) && dg::aligned(dir_enc, 16), DG_ERR_ARG, "dg_mlp_fwd: feat must be 4-byte, dir_enc 16-byte aligned");
        dg::mlp_mfma_fwd(weights, feat, dir_enc, app, desc->n_app, S, N, desc->act_c, sigma, rgb, st);
    } else
        mlp_fwd_kernel<NetTiny><<<(uint32_t)n_blocks, kFwdBlock, 0, st>>>((const __half *)weights, (const __half *)feat,
                                                                           (const __half *)dir_enc, S, N, desc->act_c, sigma, rgb);
    return dg::launch_status("dg_mlp_fwd");
}

extern "C" int dg_mlp_composite_fwd(const dg_mlp_desc *desc, const void *weights, const void *feat, const void *dir_enc,
                                    const void *app, uint32_t S, uint32_t n_seg, const float *delta, const float *t,
                                    const uint32_t *seg_ray, const uint32_t *seg_slot, uint32_t k_max, float *Ck, float *Tk,
                                    float *Dk, void *stream)
{
    const int net = which_net(desc, "dg_mlp_composite_fwd");
    if (net < 0) return net;
    DG_REQUIRE(net == 1, DG_ERR_UNSUPPORTED, "dg_mlp_composite_fwd: only the 32-64-16 / 64-64-3 networks have a fused kernel");
    DG_REQUIRE(S >= 1 && S <= 64, DG_ERR_UNSUPPORTED, "dg_mlp_composite_fwd: S=%u outside 1..64 (one wavefront renders a segment)", S);
    DG_REQUIRE(k_max >= 1, DG_ERR_ARG, "dg_mlp_composite_fwd: k_max must be >= 1");
    if (n_seg == 0) return DG_OK;
    DG_REQUIRE(weights && feat && dir_enc && delta && seg_ray && seg_slot && Ck && Tk, DG_ERR_ARG, "dg_mlp_composite_fwd: null pointer");
    DG_REQUIRE((t == nullptr) == (Dk == nullptr), DG_ERR_ARG, "dg_mlp_composite_fwd: t and Dk go together");
    DG_REQUIRE(desc->n_app == 0 || (app && dg::aligned(app, 16)), DG_ERR_ARG, "dg_mlp_composite_fwd: appearance rows missing or not 16-byte aligned");
    DG_REQUIRE(dg::aligned(feat, 4) && dg::aligned(dir_enc, 16), DG_ERR_ARG, "dg_mlp_composite_fwd: feat must be 4-byte, dir_enc 16-byte aligned");
    dg::mlp_mfma_render(weights, feat, dir_enc, app, desc->n_app, S, n_seg, desc->act_c, delta, t, seg_ray, seg_slot, k_max, Ck, Tk, Dk,
                        (hipStream_t)stream);
    return dg::launch_status("dg_mlp_composite_fwd");
}

extern "C" size_t dg_mlp_bwd_workspace_bytes(const dg_mlp_desc *desc, uint64_t N)
{
    return dg_mlp_bwd_app_workspace_bytes(desc, N, 1);
}

extern "C" size_t dg_mlp_bwd_app_workspace_bytes(const dg_mlp_desc *desc, uint64_t N, uint32_t S)
{
    if (!desc || S == 0) return 0;
    const size_t scalar = (size_t)kBwdGrid * dg_mlp_weight_count(desc) * sizeof(float);
    const bool ngp = desc->n_feat == 32 && desc->n_hidden_d == 64 && desc->n_geo == 16 && desc->n_dir == 16 &&
                     desc->n_hidden_c == 64 && desc->n_layers_c == 2;
    return ngp ? dg::mlp_mfma_workspace_bytes(N, desc->n_app, S) : scalar;
}

extern "C" int dg_mlp_bwd(const dg_mlp_desc *desc, const void *weights, const void *feat, const void *dir_enc,
                          uint32_t S, uint64_t N, const float *dsigma, const float *drgb, float loss_scale,
                          float *dfeat, float *dW, void *ws, size_t ws_bytes, void *stream)
{
    DG_REQUIRE(!desc || desc->n_app == 0, DG_ERR_ARG, "dg_mlp_bwd: a network with appearance inputs needs dg_mlp_bwd_app");
    return dg_mlp_bwd_app(desc, weights, feat, dir_enc, nullptr, S, N, dsigma, drgb, loss_scale, dfeat, dW, ws, ws_bytes, stream);
}

extern "C" int dg_mlp_bwd_app(const dg_mlp_desc *desc, const void *weights, const void *feat, const void *dir_enc,
                              const void *app, uint32_t S, uint64_t N, const float *dsigma, const float *drgb,
                              float loss_scale, float *dfeat, float *dW, void *ws, size_t ws_bytes, void *stream)
{
    const int net = which_net(desc, "dg_mlp_bwd");
    if (net < 0) return net;
    DG_REQUIRE(S >= 1 && loss_scale > 0.0f, DG_ERR_ARG, "dg_mlp_bwd: S >= 1 and loss_scale > 0 required");
    if (N == 0) return DG_OK;
    DG_REQUIRE(weights && feat && dir_enc && dsigma && drgb && dfeat && dW, DG_ERR_ARG, "dg_mlp_bwd: null pointer");
    DG_REQUIRE(desc->n_app == 0 || (app && dg::aligned(app, 16)), DG_ERR_ARG, "dg_mlp_bwd: appearance rows missing or not 16-byte aligned");
    DG_REQUIRE(ws && ws_bytes >= dg_mlp_bwd_app_workspace_bytes(desc, N, S), DG_ERR_WORKSPACE, "dg_mlp_bwd: workspace %zu < %zu bytes",
               ws_bytes, dg_mlp_bwd_app_workspace_bytes(desc, N, S));
    DG_REQUIRE(dg::aligned(ws, 256), DG_ERR_ARG, "dg_mlp_bwd: workspace must be 256-byte aligned");
    const uint64_t n_tiles = (N + kBwdBlock - 1) / kBwdBlock;
    const uint32_t grid = (uint32_t)(n_tiles < kBwdGrid ? n_tiles : kBwdGrid);
    const uint32_t n_w = (uint32_t)dg_mlp_weight_count(desc);
    hipStream_t st = (hipStream_t)stream;
    if (net == 1) {
        DG_REQUIRE(dg::aligned(feat, 4) && dg::aligned(dir_enc, 16) && dg::aligned(dfeat, 8), DG_ERR_ARG,
                   "dg_mlp_bwd: feat must be 4-byte, dfeat 8-byte, dir_enc 16-byte aligned");
        dg::mlp_mfma_bwd(weights, feat, dir_enc, app, desc->n_app, S, N, desc->act_c, dsigma, drgb, loss_scale, dfeat, dW, ws, st);
        return dg::launch_status("dg_mlp_bwd");
    }
    mlp_bwd_kernel<NetTiny><<<grid, kBwdBlock, 0, st>>>((const __half *)weights, (const __half *)feat, (const __half *)dir_enc,
                                                        S, N, desc->act_c, dsigma, drgb, loss_scale, dfeat, (float *)ws);
    fold_partials_kernel<<<(n_w + 255) / 256, 256, 0, st>>>((const float *)ws, grid, n_w, 1.0f / loss_scale, dW);
    return dg::launch_status("dg_mlp_bwd");
}
