// Shared host-side helpers of the rd library (argument checks, launch checks).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "rd.h"

#define RD_WAVE 64

static inline bool rd_aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

static inline int rd_check_launch()
{
    return hipGetLastError() == hipSuccess ? RD_OK : RD_ERR_HIP;
}

// Validates the (W, L) pair shared by rd_dedup and rd_accept.
static inline int rd_check_beam_shape(int B, int W, int L)
{
    if (B <= 0 || W <= 0 || L <= 0) return RD_ERR_INVALID_ARG;
    if (W > RD_MAX_W) return RD_ERR_UNSUPPORTED;
    if ((long long)W * (long long)L > RD_MAX_N) return RD_ERR_UNSUPPORTED;
    return RD_OK;
}
