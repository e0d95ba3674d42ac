// Pieces shared by the bf16 (MFMA) and fp32 tree-attention kernels: the split plan, the
// partial-result workspace layout and the in-kernel combine done by the last workgroup
// of a (sequence, head) to finish.
//
// Work decomposition (flash-decoding style).  The keys a packed row may see are the
// context keys 0..ctx_len-1 plus the packed keys allowed by its mask row (Sec. 3.3).  For
// each (sequence, head) the context keys are cut into S contiguous ranges and the packed
// keys form one more range; one workgroup per range computes, for all packed rows at once,
// a partial softmax state (running max m, sum l, unnormalised output O) and stores it in
// the workspace.  The workgroup that finishes last for that (sequence, head) — found with
// a device-scope counter — merges the S+1 partials, normalises and writes the output, so
// the whole operation is a single launch.
#pragma once
#include "rd_internal.h"

namespace rd {

constexpr int kAttnThreads = 256;
constexpr int kBlockKeys = 128;   // keys handled per workgroup iteration

struct AttnPlan {
    int S;             // context splits per (sequence, head); partials per head = S + 1
    int rows_pad;      // packed rows padded to a multiple of 16
    size_t counters_bytes;
    size_t partial_floats;   // floats per partial: m[rows_pad] + l[rows_pad] + O[rows_pad][D]
    size_t total_bytes;
};

static inline int env_int(const char *name, int dflt)
{
    const char *v = getenv(name);
    return (v && *v) ? atoi(v) : dflt;
}

// How many context splits: enough workgroups to cover the 256 compute units a few times
// over, never more than one split per 128-key block.
static inline AttnPlan attn_plan(int B, int H, int N, int D, int Cmax)
{
    AttnPlan p;
    const long long BH = (long long)B * H;
    const int nblk = (Cmax + kBlockKeys - 1) / kBlockKeys;
    static const int target_wgs = env_int("RD_ATTN_TARGET_WGS", 1024);
    long long S = (target_wgs + BH - 1) / BH - 1;
    if (S > nblk) S = nblk;
    if (S < 1) S = 1;
    static const int forced = env_int("RD_ATTN_SPLITS", 0);
    if (forced > 0) S = forced < nblk ? forced : (nblk > 0 ? nblk : 1);
    p.S = (int)S;
    p.rows_pad = (N + 15) / 16 * 16;
    p.counters_bytes = ((size_t)BH * sizeof(uint32_t) + 255) / 256 * 256;
    p.partial_floats = (size_t)p.rows_pad * (2 + D);
    p.total_bytes = p.counters_bytes + (size_t)BH * (p.S + 1) * p.partial_floats * sizeof(float);
    return p;
}

struct AttnArgs {
    const void *q, *k_cache, *v_cache, *k_new, *v_new;
    const int32_t *ctx_len, *n_packed;
    const uint64_t *mask_bits;
    void *out;
    uint32_t *counters;
    float *partials;
    int B, H, N, Cmax, S, words, rows_pad;
    float scale_log2e;
};

__device__ __forceinline__ int clampi(int x, int lo, int hi) { return x < lo ? lo : (x > hi ? hi : x); }

// Context key range [k_begin, k_end) of split s out of S for a context of C keys: whole
// 128-key blocks, spread as evenly as whole blocks allow.
__device__ __forceinline__ void ctx_range(int C, int S, int s, int *k_begin, int *k_end)
{
    const int nblk = (C + kBlockKeys - 1) / kBlockKeys;
    const int per = (nblk + S - 1) / S;
    const int kb = s * per * kBlockKeys;
    *k_begin = kb < C ? kb : C;
    const int ke = kb + per * kBlockKeys;
    *k_end = ke < C ? ke : C;
}

__device__ __forceinline__ void store_out4(float *dst, float a, float b, float c, float d)
{
    *reinterpret_cast<float4 *>(dst) = make_float4(a, b, c, d);
}
__device__ __forceinline__ void store_out4(__bf16 *dst, float a, float b, float c, float d)
{
    typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
    bf16x4 v;
    v[0] = (__bf16)a; v[1] = (__bf16)b; v[2] = (__bf16)c; v[3] = (__bf16)d;   // round to nearest even
    *reinterpret_cast<bf16x4 *>(dst) = v;
}

// Signals that this workgroup's partial is stored; returns true in every thread of the
// workgroup that arrives last among `expected` for this (sequence, head).
__device__ __forceinline__ bool arrive_is_last(uint32_t *counter, uint32_t expected)
{
    __shared__ uint32_t s_last;
    __threadfence();          // release: partial stores become visible device-wide
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t prev = atomicAdd(counter, 1u);
        s_last = (prev == expected - 1u) ? 1u : 0u;
    }
    __syncthreads();
    const bool last = s_last != 0u;
    if (last) __threadfence();   // acquire: see the other workgroups' partials
    return last;
}

// Merge of the S+1 partial softmax states of one (sequence, head) and final store:
// out[p] = sum_s 2^(m_s - M) O_s[p] / sum_s 2^(m_s - M) l_s[p] with M = max_s m_s (scores
// are kept in log2 units).  Rows p >= P are written as zero.  Run by one workgroup.
template <int D, typename OutT>
__device__ __forceinline__ void combine_partials(const float *part /* first partial of this head */,
                                                 int n_part, size_t partial_floats, int rows_pad,
                                                 int P, int N, OutT *out /* [N][D] of this head */)
{
    constexpr int kVecPerRow = D / 4;
    constexpr int kRowsPerPass = kAttnThreads / kVecPerRow;
    const int tid = threadIdx.x;
    const int v = tid % kVecPerRow;
    for (int p = tid / kVecPerRow; p < N; p += kRowsPerPass) {
        float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
        if (p < P) {
            float M = -INFINITY;
            for (int s = 0; s < n_part; ++s) M = fmaxf(M, part[s * partial_floats + p]);
            float denom = 0.f;
            for (int s = 0; s < n_part; ++s) {
                const float *ps = part + s * partial_floats;
                const float m = ps[p];
                if (m == -INFINITY) continue;          // that range held no visible key for row p
                const float w = __builtin_amdgcn_exp2f(m - M);
                denom += w * ps[rows_pad + p];
                const float4 o = *reinterpret_cast<const float4 *>(ps + 2 * rows_pad + (size_t)p * D + 4 * v);
                a0 += w * o.x; a1 += w * o.y; a2 += w * o.z; a3 += w * o.w;
            }
            const float inv = 1.0f / denom;
            a0 *= inv; a1 *= inv; a2 *= inv; a3 *= inv;
        }
        store_out4(out + (size_t)p * D + 4 * v, a0, a1, a2, a3);
    }
}

}  // namespace rd
