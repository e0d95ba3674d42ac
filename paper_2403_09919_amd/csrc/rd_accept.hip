// rd_accept: greedy verification (Sec. 3.4, Fig. 2) for gfx950 in one launch.
//
// Phase 1 (all workgroups): the valid logit rows (p < n_packed[b]) are cut into chunks of
// a few thousand floats; a workgroup streams one chunk with 16-byte loads and reduces it to
// (max value, smallest index attaining it), which it stores in the workspace.  This phase
// is a pure HBM stream over the valid logits.
// Phase 2 (the workgroup that finishes last for a sequence, found with a device-scope
// counter): reduces the chunk results of every row to the row's arg max, then wave 0 runs
// the per-candidate prefix match with lane w = candidate w, picks the best candidate with a
// wave-wide max on (length, -w) and writes the accepted slots and the next token.
#include "rd_internal.h"

namespace {

constexpr int kAccThreads = 256;
constexpr int kMaxChunks = 64;

struct AccPlan {
    int chunks;       // chunks per logit row
    int chunk_len;    // floats per chunk (multiple of 4)
    size_t counters_bytes;
    size_t total_bytes;
};

AccPlan acc_plan(int B, int N, int V)
{
    AccPlan p;
    int chunks = (V + 2047) / 2048;
    if (chunks > kMaxChunks) chunks = kMaxChunks;
    if (chunks < 1) chunks = 1;
    int len = (V + chunks - 1) / chunks;
    len = (len + 3) / 4 * 4;
    p.chunk_len = len;
    p.chunks = (V + len - 1) / len;
    p.counters_bytes = ((size_t)B * sizeof(uint32_t) + 255) / 256 * 256;
    p.total_bytes = p.counters_bytes + (size_t)B * N * p.chunks * sizeof(unsigned long long);
    return p;
}

// (value, index) ordering of the arg max with the smallest-index tie rule.
__device__ __forceinline__ bool better(float v, int i, float bv, int bi)
{
    return v > bv || (v == bv && i < bi);
}

__global__ __launch_bounds__(kAccThreads) void rd_accept_kernel(
    const float *__restrict__ logits, const int32_t *__restrict__ beams,
    const int32_t *__restrict__ unpack_index, const int32_t *__restrict__ n_packed,
    const int32_t *__restrict__ root_token, int W, int L, int V, int chunks, int chunk_len,
    int32_t *__restrict__ argmax_out, int32_t *__restrict__ n_accept, int32_t *__restrict__ best_beam,
    int32_t *__restrict__ best_len, int32_t *__restrict__ next_token, int32_t *__restrict__ accepted_idx,
    uint32_t *counters, unsigned long long *partial)
{
    __shared__ float s_val[kAccThreads / 64];
    __shared__ int s_idx[kAccThreads / 64];
    __shared__ int s_am[RD_MAX_N];
    __shared__ uint32_t s_last;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int chunk = blockIdx.x, p = blockIdx.y, b = blockIdx.z;
    const int N = W * L;
    int P = n_packed[b];
    P = P < 1 ? 1 : (P > N ? N : P);
    if (p >= P) return;                                   // whole workgroup: row is padding

    // ---- phase 1: this chunk's (max, first index) ------------------------------------------------
    const float *row = logits + ((size_t)b * N + p) * V;
    const int v0 = chunk * chunk_len;
    const int v1 = min(V, v0 + chunk_len);
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    if ((V & 3) == 0) {
        for (int v = v0 + tid * 4; v < v1; v += kAccThreads * 4) {   // ascending v per thread
            const float4 x = *reinterpret_cast<const float4 *>(row + v);
            if (better(x.x, v, bv, bi)) { bv = x.x; bi = v; }
            if (better(x.y, v + 1, bv, bi)) { bv = x.y; bi = v + 1; }
            if (better(x.z, v + 2, bv, bi)) { bv = x.z; bi = v + 2; }
            if (better(x.w, v + 3, bv, bi)) { bv = x.w; bi = v + 3; }
        }
    } else {
        for (int v = v0 + tid; v < v1; v += kAccThreads) {
            const float x = row[v];
            if (better(x, v, bv, bi)) { bv = x; bi = v; }
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const float ov = __shfl_xor(bv, off, 64);
        const int oi = __shfl_xor(bi, off, 64);
        if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
    }
    if (lane == 0) { s_val[wave] = bv; s_idx[wave] = bi; }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < kAccThreads / 64; ++w)
            if (better(s_val[w], s_idx[w], bv, bi)) { bv = s_val[w]; bi = s_idx[w]; }
        // The chunk result crosses workgroups (possibly XCDs, each with its own L2): store and
        // later load it with device-scope accesses and wait for the store before the counter
        // moves; a device-wide fence per workgroup would flush whole L2s and dominate the kernel.
        const unsigned long long packed = (unsigned long long)__float_as_uint(bv) | ((unsigned long long)(uint32_t)bi << 32);
        __hip_atomic_store(partial + ((size_t)b * N + p) * chunks + chunk, packed, __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        const uint32_t prev = __hip_atomic_fetch_add(counters + b, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_last = (prev == (uint32_t)(P * chunks) - 1u) ? 1u : 0u;
    }
    __syncthreads();
    if (!s_last) return;
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");

    // ---- phase 2: row arg max, then token matching ---------------------------------------------------
    for (int r = tid; r < N; r += kAccThreads) {
        int am = -1;
        if (r < P) {
            const unsigned long long *pr = partial + ((size_t)b * N + r) * chunks;
            float rv = -INFINITY;
            int ri = 0x7fffffff;
            for (int c = 0; c < chunks; ++c) {
                const unsigned long long x = __hip_atomic_load(pr + c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                const float xv = __uint_as_float((uint32_t)x);
                const int xi = (int)(uint32_t)(x >> 32);
                if (better(xv, xi, rv, ri)) { rv = xv; ri = xi; }
            }
            am = ri;
        }
        s_am[r] = am;
        argmax_out[(size_t)b * N + r] = am;
    }
    __syncthreads();
    if (tid == 0) counters[b] = 0;                        // workspace ready for the next call
    if (wave != 0) return;

    const int w = lane;
    int len = 0;
    if (w < W) {
        const int32_t *bm = beams + ((size_t)b * W + w) * L;
        const int32_t *ui = unpack_index + ((size_t)b * W + w) * L;
        bool ok = (root_token == nullptr) || (bm[0] == root_token[b]);
        int prev_slot = ui[0];
        while (ok) {
            ++len;
            if (len == L) break;
            const int slot = min(max(prev_slot, 0), N - 1);
            ok = (s_am[slot] == bm[len]);
            prev_slot = ui[len];
        }
        n_accept[(size_t)b * W + w] = len;
    }
    // best candidate: longest accepted prefix, smallest index among equals
    int key = (w < W) ? (len << 8) | (255 - w) : -1;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) key = max(key, __shfl_xor(key, off, 64));
    const int bl = key >> 8;
    const int bw = 255 - (key & 255);
    const int32_t *bui = unpack_index + ((size_t)b * W + bw) * L;
    for (int t = lane; t < L; t += 64) accepted_idx[(size_t)b * L + t] = (t < bl) ? bui[t] : -1;
    if (lane == 0) {
        best_beam[b] = bw;
        best_len[b] = bl;
        next_token[b] = (bl > 0) ? s_am[min(max(bui[bl - 1], 0), N - 1)] : root_token[b];
    }
}

}  // namespace

extern "C" size_t rd_accept_workspace(int B, int W, int L, int V)
{
    if (rd_check_beam_shape(B, W, L) != RD_OK || V <= 0) return 0;
    return acc_plan(B, W * L, V).total_bytes;
}

extern "C" int rd_accept(const float *logits, const int32_t *beams, const int32_t *unpack_index,
                         const int32_t *n_packed, const int32_t *root_token,
                         int B, int W, int L, int V,
                         int32_t *argmax_out, int32_t *n_accept, int32_t *best_beam,
                         int32_t *best_len, int32_t *next_token, int32_t *accepted_idx,
                         void *workspace, size_t workspace_bytes, void *stream)
{
    const int st = rd_check_beam_shape(B, W, L);
    if (st != RD_OK) return st;
    if (V <= 0) return RD_ERR_INVALID_ARG;
    if (B > 65535) return RD_ERR_UNSUPPORTED;
    if (!logits || !beams || !unpack_index || !n_packed || !argmax_out || !n_accept || !best_beam ||
        !best_len || !next_token || !accepted_idx)
        return RD_ERR_INVALID_ARG;
    if (!rd_aligned(logits, 16)) return RD_ERR_INVALID_ARG;
    const int N = W * L;
    const AccPlan plan = acc_plan(B, N, V);
    if (!workspace || !rd_aligned(workspace, 256) || workspace_bytes < plan.total_bytes) return RD_ERR_WORKSPACE;
    uint32_t *counters = static_cast<uint32_t *>(workspace);
    unsigned long long *partial = reinterpret_cast<unsigned long long *>(static_cast<unsigned char *>(workspace) + plan.counters_bytes);
    hipLaunchKernelGGL(rd_accept_kernel, dim3(plan.chunks, N, B), dim3(kAccThreads), 0, (hipStream_t)stream,
                       logits, beams, unpack_index, n_packed, root_token, W, L, V, plan.chunks, plan.chunk_len,
                       argmax_out, n_accept, best_beam, best_len, next_token, accepted_idx, counters, partial);
    return rd_check_launch();
}
