// rd_accept_sample: acceptance by rejection sampling (Sec. 3.4's sampling mode; speculative
// sampling applied to every candidate on the packed tree) for gfx950, two launches.
//
// Launch 1 (the HBM stream): grid (chunks, N, B); a workgroup reduces one chunk of 4096 entries of a
// valid row of the LLM's logits (scaled by 1/temperature) and of the draft model's logits to
// (maximum, sum of exp(x - maximum)) each, with all of its 16-byte loads in flight together, and
// stores the two pairs in the workspace.  Rows of slots at the last position carry no draft
// distribution and their draft half is skipped.  No atomics, no counters: the partials are
// combined in a fixed order by launch 2, so results do not depend on timing.
// Launch 2 (grid: chunks of 4096 vocabulary entries x sequences, 256 threads).  Every workgroup of a
// sequence repeats the small part: log-sum-exps of the rows from the partials; one thread per
// candidate token gathers the two logits of its token under its parent slot and decides
// u < min(1, p/q); one thread per candidate counts its accepted prefix; the best candidate is the
// longest (smallest index among equals).  The token that follows is drawn by inverting a cumulative
// distribution with the caller's uniform number.  One compute unit alone needs ~10 us for the 2 x V
// exponentials of a residual max(0, p - q), so that pass is spread: each workgroup sums the residual
// weights of its own chunk, stores the total and signals; the last one to arrive adds the totals in
// chunk order, finds the chunk in which the running total crosses the target, recomputes that
// chunk's weights and takes, by a block-wide prefix scan, the first token of positive weight whose
// cumulative weight exceeds the target.  After a fully accepted candidate the weights are p itself,
// whose chunk totals follow from launch 1's partials: workgroup 0 goes straight to the last step.
#include "rd_internal.h"
#include <math.h>

RD_TRACE_DEFINE(rd_debug_set_trace_sample)

namespace {

constexpr int kLseThreads = 256;
constexpr int kLseChunk = 4096;              // entries per workgroup of launch 1: 4 x 16 bytes per thread and array
constexpr int kSelThreads = 256;
constexpr int kSelPer = 16;                  // consecutive entries per thread of launch 2
constexpr int kSelChunk = kSelPer * kSelThreads;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kMaxSelChunks = 256;           // V <= 1 Mi entries
static_assert(kSelChunk == kLseChunk, "launch 2 takes the chunk totals of p from launch 1's partials");

// Entries v .. v+3 of a row, -inf past the end (weight 0, neutral for the maximum).  No branch: a
// load inside a branch makes the compiler wait for every load in flight at the join, which turns a
// batch of loads into a chain of round trips.  Addresses past the end are pulled back into the row
// and the values replaced afterwards.  VEC: V is a multiple of 4 (16-byte loads), else four scalar loads.
template <bool VEC>
__device__ __forceinline__ float4 load4(const float *row, int v, int V)
{
    float4 r;
    if constexpr (VEC) {
        r = *reinterpret_cast<const float4 *>(row + min(v, V - 4));
        if (v >= V) r = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
    } else {
        r.x = row[min(v, V - 1)];
        r.y = row[min(v + 1, V - 1)];
        r.z = row[min(v + 2, V - 1)];
        r.w = row[min(v + 3, V - 1)];
        if (v >= V) r.x = -INFINITY;
        if (v + 1 >= V) r.y = -INFINITY;
        if (v + 2 >= V) r.z = -INFINITY;
        if (v + 3 >= V) r.w = -INFINITY;
    }
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

// The draft model's logits of the distribution after candidate w's token j (which sits in packed
// slot `slot`): row `slot` of the packed layout [B][N][V], or, in the layout the beam search records
// ([L-1][rows_per_step][V] plus step_row [B][W][L-1]), row step_row[b][w][j] of step j.
__device__ __forceinline__ const float *draft_row_ptr(const float *draft_logits, const int32_t *step_row, int rows_per_step,
                                                      int b, int w, int j, int slot, int W, int L, int V)
{
    if (step_row == nullptr) return draft_logits + ((size_t)b * W * L + slot) * V;
    const int r = min(max(step_row[((size_t)b * W + w) * (L - 1) + j], 0), rows_per_step - 1);
    return draft_logits + ((size_t)j * rows_per_step + r) * V;
}

template <bool VEC>
__global__ __launch_bounds__(kLseThreads) void rd_lse_chunk_kernel(
    const float *__restrict__ logits, const float *__restrict__ draft_logits, const int32_t *__restrict__ step_row,
    int rows_per_step, const int32_t *__restrict__ unpack_index,
    const int32_t *__restrict__ n_packed, int W, int L, int V, int chunks, float inv_t, float4 *__restrict__ part)
{
    __shared__ float s_red[kLseThreads / 64];
    __shared__ int s_owner;
    const int tid = threadIdx.x;
    const int chunk = blockIdx.x, p = blockIdx.y, b = blockIdx.z;
    const int N = W * L;
    int P = n_packed[b];
    P = P < 1 ? 1 : (P > N ? N : P);
    if (p >= P) return;
    // which (candidate, position) this slot holds: the first entry of unpack_index that names it
    if (tid == 0) s_owner = 0x7fffffff;
    __syncthreads();
    for (int e = tid; e < N; e += kLseThreads)
        if (unpack_index[(size_t)b * N + e] == p) atomicMin(&s_owner, e);
    const size_t rowid = (size_t)b * N + p;
    const float *zp = logits + rowid * V;
    const int v0 = chunk * kLseChunk;
    float4 xp[4], xq[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) xp[u] = load4<VEC>(zp, v0 + (u * kLseThreads + tid) * 4, V);
    const float2 a = chunk_max_sum(xp, inv_t, s_red);       // (its barriers also publish s_owner)
    float2 c = make_float2(0.f, 1.f);
    const int owner = s_owner;
    const int ow = owner / L, oj = owner - ow * L;
    if (owner != 0x7fffffff && oj < L - 1) {                // uniform: not at the last position, a draft row exists
        const float *zq = draft_row_ptr(draft_logits, step_row, rows_per_step, b, ow, oj, p, W, L, V);
#pragma unroll
        for (int u = 0; u < 4; ++u) xq[u] = load4<VEC>(zq, v0 + (u * kLseThreads + tid) * 4, V);
        c = chunk_max_sum(xq, 1.0f, s_red);
    }
    if (tid == 0) part[rowid * chunks + chunk] = make_float4(a.x, a.y, c.x, c.y);
}

// weight of entry v in the distribution the next token is drawn from
__device__ __forceinline__ float weight(float zp, float zq, float inv_t, float lse_p, float lse_q, bool residual)
{
    const float p = __expf(zp * inv_t - lse_p);             // exp(-inf) = 0 past the end of the row
    if (!residual) return p;
    return fmaxf(p - __expf(zq - lse_q), 0.f);
}

// Exclusive prefix sums of one value per thread over the workgroup, in thread order; `total` gets the
// workgroup's sum (the same bits in every thread).
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

// The 16 consecutive weights of this thread in chunk `chunk` of the row; returns their sum.
template <bool VEC>
__device__ __forceinline__ float chunk_weights(const float *zp, const float *zq, int chunk, int V, float inv_t,
                                               float lse_p, float lse_q, bool residual, float (&w)[kSelPer])
{
    const int v0 = chunk * kSelChunk + threadIdx.x * kSelPer;
    const float *zr = residual ? zq : zp;                   // no draft row to read when drawing from p (value unused)
    float4 a[kSelPer / 4], q[kSelPer / 4];
#pragma unroll
    for (int i = 0; i < kSelPer / 4; ++i) a[i] = load4<VEC>(zp, v0 + 4 * i, V);
#pragma unroll
    for (int i = 0; i < kSelPer / 4; ++i) q[i] = load4<VEC>(zr, v0 + 4 * i, V);
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < kSelPer / 4; ++i) {
        w[4 * i + 0] = weight(a[i].x, q[i].x, inv_t, lse_p, lse_q, residual);
        w[4 * i + 1] = weight(a[i].y, q[i].y, inv_t, lse_p, lse_q, residual);
        w[4 * i + 2] = weight(a[i].z, q[i].z, inv_t, lse_p, lse_q, residual);
        w[4 * i + 3] = weight(a[i].w, q[i].w, inv_t, lse_p, lse_q, residual);
        sum += ((w[4 * i] + w[4 * i + 1]) + w[4 * i + 2]) + w[4 * i + 3];
    }
    return sum;
}

__device__ __forceinline__ void st_dev(float *p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ float ld_dev(const float *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

template <bool VEC>
__global__ __launch_bounds__(kSelThreads) void rd_accept_sample_kernel(
    const float *__restrict__ logits, const float *__restrict__ draft_logits, const int32_t *__restrict__ step_row,
    int rows_per_step, const int32_t *__restrict__ beams,
    const int32_t *__restrict__ unpack_index, const int32_t *__restrict__ n_packed,
    const int32_t *__restrict__ root_token, const float *__restrict__ u_accept, const float *__restrict__ u_next,
    int W, int L, int V, int chunks, float inv_t, const float4 *__restrict__ part,
    float *chunk_totals /*[B][chunks]*/, uint32_t *counters /*[B]*/,
    int32_t *__restrict__ n_accept, int32_t *__restrict__ best_beam, int32_t *__restrict__ best_len,
    int32_t *__restrict__ next_token, int32_t *__restrict__ accepted_idx)
{
    __shared__ float s_lse_p[RD_MAX_N], s_lse_q[RD_MAX_N];
    __shared__ int s_slot[RD_MAX_N];
    __shared__ unsigned char s_ok[RD_MAX_N];
    __shared__ int s_best, s_pick, s_lastpos;
    __shared__ uint32_t s_last;
    __shared__ float s_wave[kSelWaves];
    __shared__ float s_total[kMaxSelChunks];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int chunk = blockIdx.x, b = blockIdx.y;
    const int N = W * L;
    int P = n_packed[b];
    P = P < 1 ? 1 : (P > N ? N : P);
    const int my_root = root_token ? root_token[b] : 0;
    const float u_draw = u_next[b];
    RD_TR(0);

    // ---- every workgroup of the sequence: log-sum-exps, rejection tests, best candidate -------------------
    for (int r = tid; r < N; r += kSelThreads) {
        float lp = 0.f, lq = 0.f;
        if (r < P) {
            const float4 *pr = part + ((size_t)b * N + r) * chunks;
            float mp = -INFINITY, mq = -INFINITY;
            for (int c = 0; c < chunks; ++c) { mp = fmaxf(mp, pr[c].x); mq = fmaxf(mq, pr[c].z); }
            float sp = 0.f, sq = 0.f;
            for (int c = 0; c < chunks; ++c) {              // in chunk order: the same bits in every workgroup
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
    RD_TR(1);

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
                const float *zq_row = draft_row_ptr(draft_logits, step_row, rows_per_step, b, e / L, j - 1, s, W, L, V);
                const float lp = logits[((size_t)b * N + s) * V + x] * inv_t - s_lse_p[s];
                const float lq = zq_row[x] - s_lse_q[s];
                const float ratio = fminf(__expf(lp - lq), 1.0f);
                ok = u_accept[(size_t)b * N + c] < ratio;
            }
        }
        s_ok[e] = ok ? 1 : 0;
    }
    __syncthreads();
    RD_TR(2);

    // one thread per candidate: length of the accepted prefix; best = longest, then smallest index
    static_assert(RD_MAX_W <= kSelThreads && RD_MAX_W <= 256, "one thread per candidate, index in 8 bits");
    if (tid < W) {
        int len = 0;
        while (len < L && s_ok[tid * L + len]) ++len;
        if (chunk == 0) n_accept[(size_t)b * W + tid] = len;
        atomicMax(&s_best, (len << 8) | (255 - tid));
    }
    __syncthreads();
    RD_TR(3);
    const int key = s_best;
    const int bl = key >> 8, bw = 255 - (key & 255);
    if (chunk == 0) {
        for (int t = tid; t < L; t += kSelThreads) accepted_idx[(size_t)b * L + t] = (t < bl) ? s_slot[bw * L + t] : -1;
        if (tid == 0) { best_beam[b] = bw; best_len[b] = bl; }
    }
    if (bl == 0) {                                          // the first token was refuted: nothing to draw
        if (chunk == 0 && tid == 0) next_token[b] = my_root;
        return;
    }

    // ---- the next token: inverse CDF of p (whole candidate accepted) or of the residual -------------------
    const int s = s_slot[bw * L + bl - 1];
    const float *zp = logits + ((size_t)b * N + s) * V;
    // (not read when the candidate was accepted whole)
    const float *zq = bl < L ? draft_row_ptr(draft_logits, step_row, rows_per_step, b, bw, bl - 1, s, W, L, V) : zp;
    const float lse_p = s_lse_p[s], lse_q = s_lse_q[s];
    const float4 *prow = part + ((size_t)b * N + s) * chunks;
    bool residual = bl < L;
    float w[kSelPer];
    if (residual) {
        // this workgroup's chunk of the residual: total -> workspace, then find out who is last
        float t = chunk_weights<VEC>(zp, zq, chunk, V, inv_t, lse_p, lse_q, true, w);
        for (int off = 32; off > 0; off >>= 1) t += __shfl_xor(t, off, 64);
        if (lane == 0) s_wave[wave] = t;
        __syncthreads();
        if (tid == 0) {
            st_dev(chunk_totals + (size_t)b * chunks + chunk, (s_wave[0] + s_wave[1]) + (s_wave[2] + s_wave[3]));
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");          // the total is visible before the arrival
            const uint32_t prev = __hip_atomic_fetch_add(counters + b, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            s_last = (prev + 1u == (uint32_t)chunks) ? 1u : 0u;
        }
        __syncthreads();
        if (!s_last) return;
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        if (tid == 0) counters[b] = 0;                      // ready for the next call
        for (int i = tid; i < chunks; i += kSelThreads) s_total[i] = ld_dev(chunk_totals + (size_t)b * chunks + i);
        __syncthreads();
        float total = 0.f;
        for (int i = 0; i < chunks; ++i) total += s_total[i];
        if (!(total > 0.f)) residual = false;               // p == q everywhere: draw from p
        __syncthreads();
    } else if (chunk != 0) {
        return;
    }
    RD_TR(4);
    if (!residual)                                          // chunk totals of p from launch 1's partials
        for (int i = tid; i < chunks; i += kSelThreads) s_total[i] = prow[i].y * __expf(prow[i].x - lse_p);
    __syncthreads();
    float total = 0.f;
    for (int i = 0; i < chunks; ++i) total += s_total[i];
    const float target = u_draw * total;
    // the chunk in which the running total crosses the target; if rounding leaves none, the last chunk
    // that holds any weight
    int ci = -1, lastc = 0;
    float base = 0.f, run = 0.f;
    for (int i = 0; i < chunks; ++i) {
        if (s_total[i] > 0.f) lastc = i;
        const float next = run + s_total[i];
        if (ci < 0 && target < next) { ci = i; base = run; }
        run = next;
    }
    if (ci < 0) { ci = lastc; base = 0.f; }
    // cumulative weights inside the chunk, in token order.  The scan sums in another order than the
    // chunk totals did, so its last value may fall short of the target by rounding: then the chunk's
    // last token of positive weight is the one.
    const float tsum = chunk_weights<VEC>(zp, zq, ci, V, inv_t, lse_p, lse_q, residual, w);
    float chunk_total;
    float cum = base + block_exclusive_scan(tsum, s_wave, chunk_total);
    const int v0 = ci * kSelChunk + tid * kSelPer;
    int pick = 0x7fffffff, lastpos = -1;
#pragma unroll
    for (int k = 0; k < kSelPer; ++k) {
        cum += w[k];
        if (w[k] > 0.f) {
            lastpos = v0 + k;
            if (pick == 0x7fffffff && cum > target) pick = v0 + k;
        }
    }
    if (pick != 0x7fffffff) atomicMin(&s_pick, pick);
    if (lastpos >= 0) atomicMax(&s_lastpos, lastpos);
    __syncthreads();
    RD_TR(5);
    if (tid == 0) {
        int tok = s_pick;
        if (tok == 0x7fffffff) tok = s_lastpos;             // rounding left no crossing: the last token of positive weight
        if (tok < 0) tok = 0;
        next_token[b] = tok;
    }
}

struct SamplePlan {
    int chunks;
    size_t totals_off, part_off;         // byte offsets in the workspace (arrival counters at 0)
    size_t total_bytes;
};

SamplePlan sample_plan(int B, int N, int V)
{
    SamplePlan p;
    auto up = [](size_t x) { return (x + 255) / 256 * 256; };
    p.chunks = (V + kLseChunk - 1) / kLseChunk;
    p.totals_off = up((size_t)B * sizeof(uint32_t));
    p.part_off = p.totals_off + up((size_t)B * p.chunks * sizeof(float));
    p.total_bytes = p.part_off + up((size_t)B * N * p.chunks * sizeof(float4));
    return p;
}

}  // namespace

extern "C" size_t rd_accept_sample_workspace(int B, int W, int L, int V)
{
    if (rd_check_beam_shape(B, W, L) != RD_OK || V <= 0 || V > kMaxSelChunks * kSelChunk) return 0;
    return sample_plan(B, W * L, V).total_bytes;
}

extern "C" int rd_accept_sample(const float *logits, const float *draft_logits, const int32_t *draft_step_row,
                                int draft_rows_per_step, const int32_t *beams, const int32_t *unpack_index, const int32_t *n_packed, const int32_t *root_token,
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
    if (draft_step_row != nullptr && draft_rows_per_step <= 0) return RD_ERR_INVALID_ARG;
    const int N = W * L;
    const SamplePlan plan = sample_plan(B, N, V);
    if (!workspace || !rd_aligned(workspace, 256) || workspace_bytes < plan.total_bytes) return RD_ERR_WORKSPACE;
    unsigned char *ws = static_cast<unsigned char *>(workspace);
    uint32_t *counters = reinterpret_cast<uint32_t *>(ws);
    float *chunk_totals = reinterpret_cast<float *>(ws + plan.totals_off);
    float4 *part = reinterpret_cast<float4 *>(ws + plan.part_off);
    const float inv_t = 1.0f / temperature;
    hipStream_t s = (hipStream_t)stream;
    const bool vec = (V & 3) == 0;                          // rows stay 16-byte aligned
    hipLaunchKernelGGL(vec ? rd_lse_chunk_kernel<true> : rd_lse_chunk_kernel<false>, dim3(plan.chunks, N, B),
                       dim3(kLseThreads), 0, s, logits, draft_logits, draft_step_row, draft_rows_per_step, unpack_index, n_packed, W, L, V,
                       plan.chunks, inv_t, part);
    if (rd_check_launch() != RD_OK) return RD_ERR_HIP;
    hipLaunchKernelGGL(vec ? rd_accept_sample_kernel<true> : rd_accept_sample_kernel<false>, dim3(plan.chunks, B),
                       dim3(kSelThreads), 0, s, logits, draft_logits, draft_step_row, draft_rows_per_step, beams, unpack_index, n_packed,
                       root_token, u_accept,
                       u_next, W, L, V, plan.chunks, inv_t, part, chunk_totals, counters, n_accept, best_beam, best_len,
                       next_token, accepted_idx);
    return rd_check_launch();
}
