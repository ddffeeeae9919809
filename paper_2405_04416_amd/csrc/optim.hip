// Optimiser step on the trainable parameters (Sec. 5.1: Adam): one HBM sweep that reads the gradient, updates the
// parameter and both moments in place and clears the gradient for the next step.
//
// The hash tables dominate (up to a few hundred million fp32 values) and a step touches only part of them, so the
// sweep is organised around the gradient: a lane reads 16 bytes of gradient and, under the rule that untouched
// entries are left alone, lanes whose four gradients are all zero stop there -- they fetch neither the parameter nor
// the moments and write nothing.  Touched parts cost 16 B read + 16 B written per value, untouched ones 4 B read.
#include "dg_internal.h"

namespace {

constexpr int kBlock = 256;

struct AdamConst {
    float lr, beta1, beta2, eps, l2;
    float inv_c1, inv_c2;       // 1 / (1 - beta^t), from the host in double
    uint32_t skip_zero;
};

__device__ __forceinline__ void adam_one(float &theta, float g, float &m, float &v, const AdamConst &c)
{
    g += c.l2 * theta;
    m = c.beta1 * m + (1.0f - c.beta1) * g;
    v = c.beta2 * v + (1.0f - c.beta2) * g * g;
    theta -= c.lr * (m * c.inv_c1) / (sqrtf(v * c.inv_c2) + c.eps);
}

// four values per lane; the tail (n % 4 values) is handled by the first lanes of the last workgroup one by one
__global__ void __launch_bounds__(kBlock)
adam_kernel(float *__restrict__ param, float *__restrict__ grad, float *__restrict__ m, float *__restrict__ v, uint64_t n,
            AdamConst c, __half *__restrict__ param_half)
{
    const uint64_t n4 = n / 4, i = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
    if (i < n4) {
        // every array is touched once per sweep and is far larger than the caches: non-temporal loads and stores
        typedef float f4 __attribute__((ext_vector_type(4)));
        const f4 g = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(grad) + i);
        const bool touched = g.x != 0.0f || g.y != 0.0f || g.z != 0.0f || g.w != 0.0f;
        if (touched || !c.skip_zero) {
            const f4 p0 = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(param) + i);
            const f4 m0 = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(m) + i);
            const f4 v0 = __builtin_nontemporal_load(reinterpret_cast<const f4 *>(v) + i);
            float p[4] = {p0.x, p0.y, p0.z, p0.w}, mm[4] = {m0.x, m0.y, m0.z, m0.w}, vv[4] = {v0.x, v0.y, v0.z, v0.w};
            const float gg[4] = {g.x, g.y, g.z, g.w};
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if (gg[k] != 0.0f || !c.skip_zero) adam_one(p[k], gg[k], mm[k], vv[k], c);
            __builtin_nontemporal_store(f4{p[0], p[1], p[2], p[3]}, reinterpret_cast<f4 *>(param) + i);
            __builtin_nontemporal_store(f4{mm[0], mm[1], mm[2], mm[3]}, reinterpret_cast<f4 *>(m) + i);
            __builtin_nontemporal_store(f4{vv[0], vv[1], vv[2], vv[3]}, reinterpret_cast<f4 *>(v) + i);
            if (touched) __builtin_nontemporal_store(f4{0.0f, 0.0f, 0.0f, 0.0f}, reinterpret_cast<f4 *>(grad) + i);
            if (param_half) {
                __half2 *h = reinterpret_cast<__half2 *>(param_half) + 2 * i;
                h[0] = __floats2half2_rn(p[0], p[1]);
                h[1] = __floats2half2_rn(p[2], p[3]);
            }
        }
    }
    const uint64_t tail = n - 4 * n4;
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x < tail) {
        const uint64_t k = 4 * n4 + threadIdx.x;
        const float g = grad[k];
        if (g != 0.0f || !c.skip_zero) {
            float p = param[k], mm = m[k], vv = v[k];
            adam_one(p, g, mm, vv, c);
            param[k] = p; m[k] = mm; v[k] = vv;
            grad[k] = 0.0f;
            if (param_half) param_half[k] = __float2half_rn(p);
        }
    }
}

}  // namespace

extern "C" int dg_adam_step(float *param, float *grad, float *m, float *v, uint64_t n, float lr, float beta1, float beta2,
                            float eps, uint32_t step, float l2, uint32_t skip_zero_grad, void *param_half, void *stream)
{
    if (n == 0) return DG_OK;
    DG_REQUIRE(param && grad && m && v, DG_ERR_ARG, "dg_adam_step: null pointer");
    DG_REQUIRE(dg::aligned(param, 16) && dg::aligned(grad, 16) && dg::aligned(m, 16) && dg::aligned(v, 16) &&
                   dg::aligned(param_half, 8),
               DG_ERR_ARG, "dg_adam_step: arrays must be 16-byte aligned (the fp16 copy 8-byte)");
    DG_REQUIRE(step >= 1, DG_ERR_ARG, "dg_adam_step: steps count from 1");
    DG_REQUIRE(beta1 >= 0.0f && beta1 < 1.0f && beta2 >= 0.0f && beta2 < 1.0f && eps >= 0.0f, DG_ERR_ARG,
               "dg_adam_step: beta1, beta2 must lie in [0, 1) and eps must not be negative");
    AdamConst c;
    c.lr = lr; c.beta1 = beta1; c.beta2 = beta2; c.eps = eps; c.l2 = l2;
    c.inv_c1 = (float)(1.0 / (1.0 - pow((double)beta1, (double)step)));
    c.inv_c2 = (float)(1.0 / (1.0 - pow((double)beta2, (double)step)));
    c.skip_zero = skip_zero_grad ? 1u : 0u;
    const uint64_t lanes = n / 4 > 0 ? n / 4 : 1, blocks = (lanes + kBlock - 1) / kBlock;
    DG_REQUIRE(blocks <= 0x7fffffffull, DG_ERR_UNSUPPORTED, "dg_adam_step: n too large for one launch");
    adam_kernel<<<(uint32_t)blocks, kBlock, 0, (hipStream_t)stream>>>(param, grad, m, v, n, c, (__half *)param_half);
    return dg::launch_status("dg_adam_step");
}

extern "C" float dg_cosine_lr(float lr0, float lr1, uint64_t iteration, uint64_t total)
{
    const double x = (total == 0 || iteration >= total) ? 1.0 : (double)iteration / (double)total;
    return (float)((double)lr1 + 0.5 * ((double)lr0 - (double)lr1) * (1.0 + cos(3.14159265358979323846 * x)));
}
