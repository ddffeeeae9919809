// Internal helpers shared by the HIP translation units of libdistgrid (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include "distgrid.h"

namespace dg {

void set_error(const char *fmt, ...);

inline int fail(int code, const char *fmt, ...)
{
    char buf[256];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    set_error("%s", buf);
    return code;
}

inline int launch_status(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(DG_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
    return DG_OK;
}

inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

constexpr int kWave = 64;

// binned backward of the hash-grid encode (encode_bwd_binned.hip)
size_t encode_bwd_binned_workspace_bytes(const dg_grid_desc *d, uint64_t N);
int encode_bwd_binned(const dg_grid_desc *d, const float *u, const float *dfeat, uint64_t N, float *dtable, void *ws,
                      size_t ws_bytes, bool counted, hipStream_t st);
int encode_bwd_binned_count(const dg_grid_desc *d, const float *u, uint64_t N, void *ws, size_t ws_bytes, hipStream_t st);

// matrix-core path of the 32-64-16 / (32 + n_app)-64-64-3 field MLPs (mlp_mfma.hip); n_app = 0, 16 or 48
size_t mlp_mfma_workspace_bytes(uint64_t N, uint32_t n_app, uint32_t S);
size_t mlp_mfma_weight_count(uint32_t n_app);
void mlp_mfma_fwd(const void *weights, const void *feat, const void *dir_enc, const void *app, uint32_t n_app, uint32_t S,
                  uint64_t N, uint32_t act_c, float *sigma, float *rgb, hipStream_t st);
void mlp_mfma_render(const void *weights, const void *feat, const void *dir_enc, const void *app, uint32_t n_app, uint32_t S,
                     uint32_t n_seg, uint32_t act_c, const float *delta, const float *t, const uint32_t *seg_ray,
                     const uint32_t *seg_slot, uint32_t k_max, float *Ck, float *Tk, float *Dk, hipStream_t st);
void mlp_mfma_bwd(const void *weights, const void *feat, const void *dir_enc, const void *app, uint32_t n_app, uint32_t S,
                  uint64_t N, uint32_t act_c, const float *dsigma, const float *drgb, float loss_scale, float *dfeat, float *dW,
                  void *ws, hipStream_t st);

}  // namespace dg

#define DG_REQUIRE(cond, code, ...)                     \
    do {                                                \
        if (!(cond)) return dg::fail(code, __VA_ARGS__); \
    } while (0)
