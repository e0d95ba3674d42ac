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

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every global
// load and store the wave has in flight, which turns each barrier after a global store into a
// round trip to memory.
__device__ __forceinline__ void rd_lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Validates the (W, L) pair shared by rd_dedup and rd_accept.
static inline int rd_check_beam_shape(int B, int W, int L)
{
    if (B <= 0 || W <= 0 || L <= 0) return RD_ERR_INVALID_ARG;
    if (W > RD_MAX_W) return RD_ERR_UNSUPPORTED;
    if ((long long)W * (long long)L > RD_MAX_N) return RD_ERR_UNSUPPORTED;
    return RD_OK;
}

// Optional phase timestamps for tuning builds (-DRD_TRACE): thread 0 of every workgroup stores
// the constant-rate wall clock at a few points into a caller-supplied buffer (one per source file).
#ifdef RD_TRACE
#define RD_TRACE_DEFINE(setter)                                                                   \
    __device__ unsigned long long *rd_trace_buf = nullptr;                                        \
    extern "C" int setter(unsigned long long *p)                                                  \
    {                                                                                             \
        return hipMemcpyToSymbol(HIP_SYMBOL(rd_trace_buf), &p, sizeof(p)) == hipSuccess ? 0 : -4; \
    }
#define RD_TR(i)                                                                                                   \
    do {                                                                                                           \
        if (threadIdx.x == 0 && rd_trace_buf)                                                                      \
            rd_trace_buf[((size_t)blockIdx.x + (size_t)gridDim.x * (blockIdx.y + (size_t)gridDim.y * blockIdx.z)) * 16 + (i)] = wall_clock64(); \
    } while (0)
#else
#define RD_TRACE_DEFINE(setter)
#define RD_TR(i) do { } while (0)
#endif
