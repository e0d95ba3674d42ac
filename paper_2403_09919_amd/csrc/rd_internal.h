// Shared helpers of the rd library: argument and launch checks, tuning overrides, and the
// device-scope accesses with which workgroups hand partial results to one another.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>
#include <atomic>
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

namespace rd {

// Integer environment override for tuning sweeps (unset or empty: the default).  Only builds made
// with -DRD_TUNING read the environment; in the product library every plan is fixed by its arguments.
static inline int env_int(const char *name, int dflt)
{
#ifdef RD_TUNING
    const char *v = getenv(name);
    return (v && *v) ? atoi(v) : dflt;
#else
    (void)name;
    return dflt;
#endif
}

// Raising a kernel's dynamic LDS limit is per kernel and per device; `done` (one per kernel) keeps
// a bit for each device already set up.  Returns RD_OK or RD_ERR_HIP.
static inline int ensure_dynamic_lds(const void *kernel, size_t bytes, std::atomic<unsigned long long> &done)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return RD_ERR_HIP;
    const unsigned long long bit = 1ull << (dev & 63);
    if (dev < 64 && (done.load(std::memory_order_acquire) & bit)) return RD_OK;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess)
        return RD_ERR_HIP;
    if (dev < 64) done.fetch_or(bit, std::memory_order_release);
    return RD_OK;
}

// ---- exchange of partial results between workgroups -------------------------------------------
// Partial results (attention states, K-split sums of the drafter's layers) are written by one
// workgroup and read by another that may sit on a different XCD (each XCD has its own L2).  A
// device-wide release/acquire fence would write back and invalidate whole L2s on every
// workgroup, which costs far more than the kernel itself, so the
// exchange uses device-scope (write-through / cache-bypassing) relaxed atomic accesses for the
// data itself, made complete with a wait for outstanding memory operations before the counter
// is bumped.  Only these few KB per workgroup travel that way; the bulk streams use plain loads.
__device__ __forceinline__ void st_dev(float *p, float v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_dev2(float *p, float a, float b)
{
    unsigned long long u = (unsigned long long)__float_as_uint(a) | ((unsigned long long)__float_as_uint(b) << 32);
    __hip_atomic_store(reinterpret_cast<unsigned long long *>(p), u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_dev(const float *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2 ld_dev2(const float *p)
{
    const unsigned long long u =
        __hip_atomic_load(reinterpret_cast<const unsigned long long *>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return make_float2(__uint_as_float((unsigned)u), __uint_as_float((unsigned)(u >> 32)));
}

// 16 bytes as two 8-byte device-scope stores (write-through).  Both are ordinary atomic stores the
// compiler sees, so it inserts whatever wait states the data registers need before they are reused.
__device__ __forceinline__ void st_dev4(float *p, float a, float b, float c, float d)
{
    st_dev2(p, a, b);
    st_dev2(p + 2, c, d);
}
// Returns once every vector memory operation this wave has issued -- loads, stores and atomics without
// a return value alike, they share one counter -- has been acknowledged.  A device-scope store or atomic
// is acknowledged when it has been performed past the XCD's L2, where every other XCD can see it.  This
// is the release half of the exchange; a release FENCE at device scope would also write back the whole
// L2, which is what the exchange avoids.
__device__ __forceinline__ void wait_dev_stores() { asm volatile("s_waitcnt vmcnt(0)" : : : "memory"); }

}  // namespace rd

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
