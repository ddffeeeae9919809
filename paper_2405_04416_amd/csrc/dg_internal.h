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

}  // namespace dg

#define DG_REQUIRE(cond, code, ...)                     \
    do {                                                \
        if (!(cond)) return dg::fail(code, __VA_ARGS__); \
    } while (0)
