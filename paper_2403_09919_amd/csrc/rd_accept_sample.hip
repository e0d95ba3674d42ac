// rd_accept_sample: acceptance by rejection sampling (Sec. 3.4's sampling mode; speculative
// sampling applied to every candidate on the packed tree) for gfx950, two launches.
//
// Launch 1 (the HBM stream): grid (chunks, N, B); a workgroup reduces one chunk of 4096 entries of a
// valid row of the LLM's logits (scaled by 1/temperature) and of the draft model's logits to
// (maximum, sum of exp(x - maximum)) each, with all of its 16-byte loads in flight together, and
// stores the two pairs in the workspace.  Rows of slots at the last position carry no draft
// distribution and their draft half is skipped.  No atomics, no counters: the partials are
// combined in a fixed order by launch 2, so results do not depend on timing.
// Launch 2 (one workgroup of 1024 threads per sequence): log-sum-exps of the rows; one thread per
// candidate token gathers the two logits of its token under its parent slot and decides
// u < min(1, p/q); one thread per candidate counts its accepted prefix; the best candidate is the
// longest (smallest index among equals).  The token that follows is drawn by inverting the
// cumulative distribution of p, or of the residual max(0, p - q) after a rejection, with the
// caller's uniform number: a first pass over the row computes the total of every chunk of 4096
// weights with a block-wide scan, the chunk in which the running total crosses the target is
// scanned again (same arithmetic, same values), and the first token of positive weight whose
// cumulative weight exceeds the target is taken.
#include "rd_internal.h"
#include <math.h>

namespace {

constexpr int kLseThreads = 256;
constexpr int kLseChunk = 4096;              // entries per workgroup of launch 1: 4 x 16 bytes per thread and array
constexpr int kSelThreads = 1024;
constexpr int kSelChunk = 4 * kSelThreads;   // weights per block-wide scan of launch 2
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kMaxSelChunks = 256;           // V <= 1 Mi entries

__device__ __forceinline__ float4 load4(const float *row, int v, int V, bool vec)
{
    // entries v .. v+3 of a row; -inf past the end (weight 0, neutral for the maximum)
    if (vec && v + 3 < V) return *reinterpret_cast<const float4 *>(row + v);
    float4 r;
    r.x = v < V ? row[v] : -INFINITY;
    r.y = v + 1 < V ? row[v + 1] : -INFINITY;
    r.z = v + 2 < V ? row[v + 2] : -INFINITY;
    r.w = v + 3 < V ? row[v + 3] : -INFINITY;
    return r;
}

// (maximum, sum exp(x*scale - maximum)) of up to 16 values per thread over the workgroup
__device__ __forceinline__ float2 chunk_max_sum(const float4 (&x)[4], float scale, float *s_red)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float m = -INFINITY;
#pragma unroll
    for (int u = 0; u < 4; ++u) m = fmaxf(fmaxf(fmaxf(x[u].x, x[u].y), fmaxf(x[u].z, x[u].w)) * scale, m);
    for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
    if (lane == 0) s_red[wave] = m;
    __syncthreads();
    m = fmaxf(fmaxf(s_red[0], s_red[1]), fmaxf(s_red[2], s_red[3]));
    __syncthreads();
    float s = 0.f;
    if (m > -INFINITY) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
            s += __expf(x[u].x * scale - m) + __expf(x[u].y * scale - m) + __expf(x[u].z * scale - m) + __expf(x[u].w * scale - m);
    }
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
    if (lane == 0) s_red[wave] = s;
    __syncthreads();
    s = (s_red[0] + s_red[1]) + (s_red[2] + s_red[3]);
    __syncthreads();
    return make_float2(m, s);
}

__global__ __launch_bounds__(kLseThreads) void rd_lse_chunk_kernel(
    const float *__restrict__ logits, const float *__restrict__ draft_logits, const int32_t *__restrict__ unpack_index,
    const int32_t *__restrict__ n_packed, int W, int L, int V, int chunks, float inv_t, float4 *__restrict__ part)
{
    __shared__ float s_red[kLseThreads / 64];
    __shared__ int s_leaf;
    const int tid = threadIdx.x;
    const int chunk = blockIdx.x, p = blockIdx.y, b = blockIdx.z;
    const int N = W * L;
    int P = n_packed[b];
    P = P < 1 ? 1 : (P > N ? N : P);
    if (p >= P) return;
    if (tid == 0) s_leaf = 0;
    __syncthreads();
    if (tid < W && unpack_index[(size_t)b * N + tid * L + (L - 1)] == p) s_leaf = 1;   // a slot at the last position
    const bool vec = (V & 3) == 0;
    const size_t rowid = (size_t)b * N + p;
    const float *zp = logits + rowid * V, *zq = draft_logits + rowid * V;
    const int v0 = chunk * kLseChunk;
    float4 xp[4], xq[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) xp[u] = load4(zp, v0 + (u * kLseThreads + tid) * 4, V, vec);
    __syncthreads();
    const bool leaf = s_leaf != 0;
    if (!leaf) {
#pragma unroll
        for (int u = 0; u < 4; ++u) xq[u] = load4(zq, v0 + (u * kLseThreads + tid) * 4, V, vec);
    } else {
#pragma unroll
        for (int u = 0; u < 4; ++u) xq[u] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    const float2 a = chunk_max_sum(xp, inv_t, s_red);
    const float2 c = chunk_max_sum(xq, 1.0f, s_red);
    if (tid == 0) part[rowid * chunks + chunk] = make_float4(a.x, a.y, c.x, c.y);
}

// weight of entry v in the distribution the next token is drawn from
__device__ __forceinline__ float weight(float zp, float zq, float inv_t, float lse_p, float lse_q, bool residual)
{
    const float p = __expf(zp * inv_t - lse_p);             // exp(-inf) = 0 past the end of the row
    if (!residual) return p;
    return fmaxf(p - __expf(zq - lse_q), 0.f);
}

// Inclusive prefix sums of one value per thread over the workgroup, in thread order; returns the
// exclusive prefix of this thread and, in `total`, the workgroup's sum (the same bits in every thread).
__device__ __forceinline__ float block_exclusive_scan(float x, float *s_wave, float &total)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    float incl = x;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const float o = __shfl_up(incl, off, 64);
        if (lane >= off) incl += o;
    }
    __syncthreads();                                        // s_wave free again
    if (lane == 63) s_wave[wave] = incl;
    __syncthreads();
    float before = 0.f, all = 0.f;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) {
        const float t = s_wave[w];
        if (w < wave) before += t;
        all += t;
    }
    total = all;
    return before + (incl - x);
}

__global__ __launch_bounds__(kSelThreads) void rd_accept_sample_kernel(
    const float *__restrict__ logits, const float *__restrict__ draft_logits, const int32_t *__restrict__ beams,
    const int32_t *__restrict__ unpack_index, const int32_t *__restrict__ n_packed,
    const int32_t *__restrict__ root_token, const float *__restrict__ u_accept, const float *__restrict__ u_next,
    int W, int L, int V, int chunks, float inv_t, const float4 *__restrict__ part,
    int32_t *__restrict__ n_accept, int32_t *__restrict__ best_beam, int32_t *__restrict__ best_len,
    int32_t *__restrict__ next_token, int32_t *__restrict__ accepted_idx)
{
    __shared__ float s_lse_p[RD_MAX_N], s_lse_q[RD_MAX_N];
    __shared__ int s_slot[RD_MAX_N];
    __shared__ unsigned char s_ok[RD_MAX_N];
    __shared__ int s_best, s_pick, s_lastpos;
    __shared__ float s_wave[kSelWaves];
    __shared__ float s_chunk_total[kMaxSelChunks];

    const int tid = threadIdx.x, b = blockIdx.x;
    const int N = W * L;
    int P = n_packed[b];
    P = P < 1 ? 1 : (P > N ? N : P);
    const int my_root = root_token ? root_token[b] : 0;

    // log-sum-exp of every valid row from its chunk partials, in chunk order
    for (int r = tid; r < N; r += kSelThreads) {
        float lp = 0.f, lq = 0.f;
        if (r < P) {
            const float4 *pr = part + ((size_t)b * N + r) * chunks;
            float mp = -INFINITY, mq = -INFINITY;
            for (int c = 0; c < chunks; ++c) { mp = fmaxf(mp, pr[c].x); mq = fmaxf(mq, pr[c].z); }
            float sp = 0.f, sq = 0.f;
            for (int c = 0; c < chunks; ++c) {
                const float4 v = pr[c];
                sp += v.y * __expf(v.x - mp);
                sq += v.w * __expf(v.z - mq);
            }
            lp = mp + __logf(sp);
            lq = mq + __logf(sq);
        }
        s_lse_p[r] = lp;
        s_lse_q[r] = lq;
        s_slot[r] = min(max(unpack_index[(size_t)b * N + r], 0), N - 1);
    }
    if (tid == 0) { s_best = -1; s_pick = 0x7fffffff; s_lastpos = -1; }
    __syncthreads();

    // one thread per candidate token: the rejection test of token (w, j), j >= 1
    for (int e = tid; e < N; e += kSelThreads) {
        const int j = e % L;
        const int x = beams[(size_t)b * N + e];
        bool ok;
        if (j == 0) {
            ok = (root_token == nullptr) || (x == my_root);
        } else {
            ok = false;
            if (x >= 0 && x < V) {
                const int s = s_slot[e - 1], c = s_slot[e];
                const size_t row = ((size_t)b * N + s) * V;
                const float lp = logits[row + x] * inv_t - s_lse_p[s];
                const float lq = draft_logits[row + x] - s_lse_q[s];
                const float ratio = fminf(__expf(lp - lq), 1.0f);
                ok = u_accept[(size_t)b * N + c] < ratio;
            }
        }
        s_ok[e] = ok ? 1 : 0;
    }
    __syncthreads();

    // one thread per candidate: length of the accepted prefix; best = longest, then smallest index
    static_assert(RD_MAX_W <= 256, "candidate index in 8 bits");
    if (tid < W) {
        int len = 0;
        while (len < L && s_ok[tid * L + len]) ++len;
        n_accept[(size_t)b * W + tid] = len;
        atomicMax(&s_best, (len << 8) | (255 - tid));
    }
    __syncthreads();
    const int key = s_best;
    const int bl = key >> 8, bw = 255 - (key & 255);
    for (int t = tid; t < L; t += kSelThreads) accepted_idx[(size_t)b * L + t] = (t < bl) ? s_slot[bw * L + t] : -1;
    if (tid == 0) { best_beam[b] = bw; best_len[b] = bl; }
    if (bl == 0) {                                          // the first token was refuted: nothing to draw
        if (tid == 0) next_token[b] = my_root;
        return;
    }

    // ---- the next token: inverse CDF of p (whole candidate accepted) or of the residual -------------------
    const int s = s_slot[bw * L + bl - 1];
    const float *zp = logits + ((size_t)b * N + s) * V;
    const float *zq = draft_logits + ((size_t)b * N + s) * V;       // not read when the candidate was accepted whole
    const float lse_p = s_lse_p[s], lse_q = s_lse_q[s];
    const bool vec = (V & 3) == 0;
    const int n_chunks = (V + kSelChunk - 1) / kSelChunk;
    bool residual = bl < L;
    float total = 0.f;
    for (int attempt = 0; attempt < 2; ++attempt) {
        int lastpos = -1;
        for (int i = 0; i < n_chunks; ++i) {
            const int v = i * kSelChunk + tid * 4;
            const float4 a = load4(zp, v, V, vec);
            const float4 q = residual ? load4(zq, v, V, vec) : make_float4(0.f, 0.f, 0.f, 0.f);
            const float w0 = weight(a.x, q.x, inv_t, lse_p, lse_q, residual), w1 = weight(a.y, q.y, inv_t, lse_p, lse_q, residual);
            const float w2 = weight(a.z, q.z, inv_t, lse_p, lse_q, residual), w3 = weight(a.w, q.w, inv_t, lse_p, lse_q, residual);
            if (w3 > 0.f) lastpos = v + 3; else if (w2 > 0.f) lastpos = v + 2; else if (w1 > 0.f) lastpos = v + 1; else if (w0 > 0.f) lastpos = v;
            float chunk_total;
            block_exclusive_scan(((w0 + w1) + w2) + w3, s_wave, chunk_total);
            if (tid == 0) s_chunk_total[i] = chunk_total;
        }
        if (lastpos >= 0) atomicMax(&s_lastpos, lastpos);
        __syncthreads();
        total = 0.f;
        for (int i = 0; i < n_chunks; ++i) total += s_chunk_total[i];
        if (total > 0.f || !residual) break;
        residual = false;                                   // p == q everywhere: draw from p
        __syncthreads();
        if (tid == 0) s_lastpos = -1;
        __syncthreads();
    }
    const float target = u_next[b] * total;
    // the chunk in which the running total crosses the target
    int ci = -1;
    float base = 0.f;
    for (int i = 0; i < n_chunks; ++i) {
        const float next = base + s_chunk_total[i];
        if (target < next) { ci = i; break; }
        base = next;
    }
    if (ci >= 0) {
        const int v = ci * kSelChunk + tid * 4;
        const float4 a = load4(zp, v, V, vec);
        const float4 q = residual ? load4(zq, v, V, vec) : make_float4(0.f, 0.f, 0.f, 0.f);
        const float w0 = weight(a.x, q.x, inv_t, lse_p, lse_q, residual), w1 = weight(a.y, q.y, inv_t, lse_p, lse_q, residual);
        const float w2 = weight(a.z, q.z, inv_t, lse_p, lse_q, residual), w3 = weight(a.w, q.w, inv_t, lse_p, lse_q, residual);
        float chunk_total;
        const float excl = base + block_exclusive_scan(((w0 + w1) + w2) + w3, s_wave, chunk_total);
        const float c0 = excl + w0, c1 = c0 + w1, c2 = c1 + w2, c3 = c2 + w3;
        int pick = 0x7fffffff, lastc = -1;
        if (w3 > 0.f) { lastc = v + 3; if (c3 > target) pick = v + 3; }
        if (w2 > 0.f) { lastc = max(lastc, v + 2); if (c2 > target) pick = v + 2; }
        if (w1 > 0.f) { lastc = max(lastc, v + 1); if (c1 > target) pick = v + 1; }
        if (w0 > 0.f) { lastc = max(lastc, v); if (c0 > target) pick = v; }
        __syncthreads();
        if (tid == 0) s_lastpos = -1;                       // now: last positive weight of this chunk
        __syncthreads();
        if (pick != 0x7fffffff) atomicMin(&s_pick, pick);
        if (lastc >= 0) atomicMax(&s_lastpos, lastc);
        __syncthreads();
    }
    if (tid == 0) {
        int tok = s_pick;
        if (tok == 0x7fffffff) tok = s_lastpos;             // rounding left no crossing: the last token of positive weight
        if (tok < 0) tok = 0;
        next_token[b] = tok;
    }
}

struct SamplePlan {
    int chunks;
    size_t total_bytes;
};

SamplePlan sample_plan(int B, int N, int V)
{
    SamplePlan p;
    p.chunks = (V + kLseChunk - 1) / kLseChunk;
    p.total_bytes = ((size_t)B * N * p.chunks * sizeof(float4) + 255) / 256 * 256;
    return p;
}

}  // namespace

extern "C" size_t rd_accept_sample_workspace(int B, int W, int L, int V)
{
    if (rd_check_beam_shape(B, W, L) != RD_OK || V <= 0 || V > kMaxSelChunks * kSelChunk) return 0;
    return sample_plan(B, W * L, V).total_bytes;
}

extern "C" int rd_accept_sample(const float *logits, const float *draft_logits, const int32_t *beams,
                                const int32_t *unpack_index, const int32_t *n_packed, const int32_t *root_token,
                                const float *u_accept, const float *u_next, float temperature,
                                int B, int W, int L, int V,
                                int32_t *n_accept, int32_t *best_beam, int32_t *best_len, int32_t *next_token,
                                int32_t *accepted_idx, void *workspace, size_t workspace_bytes, void *stream)
{
    const int st = rd_check_beam_shape(B, W, L);
    if (st != RD_OK) return st;
    if (V <= 0 || !(temperature > 0.f) || !isfinite(temperature)) return RD_ERR_INVALID_ARG;
    if (B > 65535 || V > kMaxSelChunks * kSelChunk) return RD_ERR_UNSUPPORTED;
    if (!logits || !draft_logits || !beams || !unpack_index || !n_packed || !u_accept || !u_next || !n_accept ||
        !best_beam || !best_len || !next_token || !accepted_idx)
        return RD_ERR_INVALID_ARG;
    if (!rd_aligned(logits, 16) || !rd_aligned(draft_logits, 16)) return RD_ERR_INVALID_ARG;
    const int N = W * L;
    const SamplePlan plan = sample_plan(B, N, V);
    if (!workspace || !rd_aligned(workspace, 256) || workspace_bytes < plan.total_bytes) return RD_ERR_WORKSPACE;
    float4 *part = static_cast<float4 *>(workspace);
    const float inv_t = 1.0f / temperature;
    hipStream_t s = (hipStream_t)stream;
    hipLaunchKernelGGL(rd_lse_chunk_kernel, dim3(plan.chunks, N, B), dim3(kLseThreads), 0, s, logits, draft_logits,
                       unpack_index, n_packed, W, L, V, plan.chunks, inv_t, part);
    if (rd_check_launch() != RD_OK) return RD_ERR_HIP;
    hipLaunchKernelGGL(rd_accept_sample_kernel, dim3(B), dim3(kSelThreads), 0, s, logits, draft_logits, beams,
                       unpack_index, n_packed, root_token, u_accept, u_next, W, L, V, plan.chunks, inv_t, part,
                       n_accept, best_beam, best_len, next_token, accepted_idx);
    return rd_check_launch();
}
