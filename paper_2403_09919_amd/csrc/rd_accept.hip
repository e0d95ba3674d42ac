// rd_accept: greedy verification (Sec. 3.4, Fig. 2) for gfx950 in one launch.
//
// Phase 1 (all workgroups): the valid logit rows (p < n_packed[b]) are cut into chunks of
// a few thousand floats; a workgroup streams one chunk with 16-byte loads, reduces it to
// (max value, smallest index attaining it) and folds that into the row's 64-bit key in the
// workspace with one device-scope atomic max.  The key orders (value, -index), so the row's
// final key is its arg max with the smallest-index tie rule.  This phase is a pure HBM stream
// over the valid logits.
// Phase 2 (the workgroup that completes a sequence, found with a per-row and then a
// per-sequence counter): decodes the row keys, writes the arg maxes, and wave 0 runs the
// per-candidate prefix match with lane w = candidate w, picks the best candidate with a
// wave-wide max on (length, -w) and writes the accepted slots and the next token.
// Two counter levels keep the number of atomics that hit one address small (chunks per row,
// rows per sequence); hundreds of increments of a single word would serialise and cost more
// than the stream itself.
#include "rd_internal.h"
#include <cstdlib>

RD_TRACE_DEFINE(rd_debug_set_trace_accept)

namespace {

constexpr int kAccThreads = 256;
constexpr int kMaxChunks = 64;

struct AccPlan {
    int chunks;       // chunks per logit row
    int chunk_len;    // floats per chunk (multiple of 1024)
    int loads;        // 16-byte loads per thread issued together (1, 2, 4, ..., 32)
    int speculate;    // 1: first loads before the packed count is known (small logit tensors)
    size_t row_counters_off, keys_off;   // byte offsets in the workspace (sequence counters at 0)
    size_t total_bytes;                  // all of it must be zero between calls (and is left so)
};

// A workgroup issues all loads of its chunk at once: `loads` 16-byte loads per thread, so a chunk
// is 1024*loads floats.  Measured on MI355X (V = 32000): 4 or 8 loads per thread (8 or 4 chunks per
// row) are best from 22 to 500 valid rows -- 6.6 us and 21 us per launch against 10.6 us and 54 us
// with one load per thread, where the extra workgroups and the 32 atomics per row dominate, and
// 10 us and 27 us with one workgroup per row, where a workgroup's own streaming rate does.
AccPlan acc_plan(int B, int N, int V)
{
    AccPlan p;
    static const int loads_env = rd::env_int("RD_ACCEPT_LOADS", 0);      // tuning builds only
    int loads = ((long long)B * N >= 512) ? 8 : 4;
    if (loads_env == 1 || loads_env == 2 || loads_env == 4 || loads_env == 8 || loads_env == 16 || loads_env == 32) loads = loads_env;
    while ((V + 1024 * loads - 1) / (1024 * loads) > kMaxChunks) loads *= 2;     // huge vocabularies: the kernel loops
    p.loads = loads > 32 ? 32 : loads;
    static const int spec_env = rd::env_int("RD_ACCEPT_SPEC", -1);       // tuning builds only
    p.speculate = ((double)B * N * V * sizeof(float) <= 8e6 && p.loads <= 8) ? 1 : 0;
    if (spec_env >= 0) p.speculate = spec_env ? 1 : 0;
    int len = 1024 * loads;
    p.chunk_len = len;
    p.chunks = (V + len - 1) / len;
    auto up = [](size_t x) { return (x + 255) / 256 * 256; };
    p.row_counters_off = up((size_t)B * sizeof(uint32_t));
    p.keys_off = p.row_counters_off + up((size_t)B * N * sizeof(uint32_t));
    p.total_bytes = p.keys_off + up((size_t)B * N * sizeof(unsigned long long));
    return p;
}

// (value, index) ordering of the arg max with the smallest-index tie rule.
__device__ __forceinline__ bool better(float v, int i, float bv, int bi)
{
    return v > bv || (v == bv && i < bi);
}

// Order-preserving 64-bit key of (value, index): larger value first, then smaller index.
// Every key of a real element is greater than 0, the cleared state of the workspace.
// -0.0 and +0.0 are one value to the comparison that defines the arg max, so both get +0.0's key.
__device__ __forceinline__ unsigned long long encode_key(float v, int i)
{
    const uint32_t u = (v == 0.0f) ? 0u : __float_as_uint(v);
    const uint32_t mono = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
    return ((unsigned long long)mono << 32) | (uint32_t)~(uint32_t)i;
}
__device__ __forceinline__ int key_index(unsigned long long k) { return (int)~(uint32_t)k; }

// Device-scope arrival: true for the thread whose increment brought the counter to `expected`.
// The thread's earlier device-scope atomics (the row key's max, a lower-level counter) and stores must
// have been performed before the counter moves: they go to other addresses and could otherwise
// complete after it, and the workgroup that sees the full count would read a key that lacks this
// workgroup's chunk.  wait_dev_stores() waits for their acknowledgement.
__device__ __forceinline__ bool arrive(uint32_t *counter, uint32_t expected)
{
    rd::wait_dev_stores();
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    const uint32_t prev = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
    return prev + 1u == expected;
}

// SPEC: the first batch of logit loads is issued before n_packed[b] is known (every row of the [B,N,V] tensor is
// allocated, so a row beyond the packed count is read and dropped): one dependent round trip less in front
// of the stream.  For launches whose whole logit tensor is a few MB, where the extra rows cost nothing.
template <int U, bool SPEC>
__global__ __launch_bounds__(kAccThreads) void rd_accept_kernel(
    const float *__restrict__ logits, const int32_t *__restrict__ beams,
    const int32_t *__restrict__ unpack_index, const int32_t *__restrict__ n_packed,
    const int32_t *__restrict__ root_token, int W, int L, int V, int chunks, int chunk_len,
    int32_t *__restrict__ argmax_out, int32_t *__restrict__ n_accept, int32_t *__restrict__ best_beam,
    int32_t *__restrict__ best_len, int32_t *__restrict__ next_token, int32_t *__restrict__ accepted_idx,
    uint32_t *seq_counters, uint32_t *row_counters, unsigned long long *row_keys)
{
    __shared__ float s_val[kAccThreads / 64];
    __shared__ int s_idx[kAccThreads / 64];
    __shared__ int s_am[RD_MAX_N];
    __shared__ int s_beam[RD_MAX_N], s_slot[RD_MAX_N];
    __shared__ uint32_t s_seq_last;
    __shared__ int s_best;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int chunk = blockIdx.x, p = blockIdx.y, b = blockIdx.z;
    const int N = W * L;
    const float *row = logits + ((size_t)b * N + p) * V;
    const int v0 = chunk * chunk_len;
    const int v1 = min(V, v0 + chunk_len);
    float4 x0[U];
    if (SPEC && (V & 3) == 0) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int v = v0 + (u * kAccThreads + tid) * 4;
            x0[u] = *reinterpret_cast<const float4 *>(row + (v < v1 ? v : v0));
        }
    }
    int P = n_packed[b];
    P = P < 1 ? 1 : (P > N ? N : P);
    if (p >= P) return;                                   // whole workgroup: row is padding
    RD_TR(0);

    // The candidates and their slots are only needed by the workgroup that ends up finishing the
    // sequence, but nobody knows which one that is: every workgroup fetches them now (a few
    // hundred bytes, overlapped with the logit stream) instead of paying two dependent round
    // trips to memory per accepted token at the very end.
    constexpr int kPre = (RD_MAX_N + kAccThreads - 1) / kAccThreads;     // tokens per thread
    int my_beam[kPre], my_slot[kPre], my_root = 0;
#pragma unroll
    for (int u = 0; u < kPre; ++u) {
        const int e = min(u * kAccThreads + tid, N - 1);
        my_beam[u] = beams[(size_t)b * N + e];
        my_slot[u] = unpack_index[(size_t)b * N + e];
    }
    if (root_token != nullptr) my_root = root_token[b];

    // ---- phase 1: this chunk's (max, first index) -> the row's key ---------------------------------
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    if ((V & 3) == 0) {
        // U loads per thread in flight together; a load past the end of the chunk is redirected to
        // the chunk's first vector and ignored, so that no load depends on a branch.
        for (int base = v0; base < v1; base += kAccThreads * 4 * U) {
            float4 x[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int v = base + (u * kAccThreads + tid) * 4;
                if (SPEC && base == v0) x[u] = x0[u];
                else x[u] = *reinterpret_cast<const float4 *>(row + (v < v1 ? v : v0));
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {                              // ascending v per thread
                const int v = base + (u * kAccThreads + tid) * 4;
                if (v < v1) {
                    if (better(x[u].x, v, bv, bi)) { bv = x[u].x; bi = v; }
                    if (better(x[u].y, v + 1, bv, bi)) { bv = x[u].y; bi = v + 1; }
                    if (better(x[u].z, v + 2, bv, bi)) { bv = x[u].z; bi = v + 2; }
                    if (better(x[u].w, v + 3, bv, bi)) { bv = x[u].w; bi = v + 3; }
                }
            }
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
    RD_TR(1);
    if (lane == 0) { s_val[wave] = bv; s_idx[wave] = bi; }
    __syncthreads();
    const size_t rowid = (size_t)b * N + p;
    if (tid == 0) {
        for (int w = 1; w < kAccThreads / 64; ++w)
            if (better(s_val[w], s_idx[w], bv, bi)) { bv = s_val[w]; bi = s_idx[w]; }
        uint32_t last = 0;
        if (bi != 0x7fffffff)                               // (an empty chunk cannot occur, but would add nothing)
            __hip_atomic_fetch_max(row_keys + rowid, encode_key(bv, bi), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (chunks == 1) {                                             // the row is this workgroup's alone
            last = arrive(seq_counters + b, (uint32_t)P) ? 1u : 0u;
        } else if (arrive(row_counters + rowid, (uint32_t)chunks)) {   // this row is complete
            row_counters[rowid] = 0;                                   // ready for the next call
            last = arrive(seq_counters + b, (uint32_t)P) ? 1u : 0u;    // ... and so is the sequence
        }
        s_seq_last = last;
    }
    RD_TR(2);
    __syncthreads();
    if (!s_seq_last) return;
    RD_TR(3);

    // ---- phase 2 (last workgroup of the sequence): arg maxes, then token matching -----------------------
    for (int r = tid; r < N; r += kAccThreads) {
        int am = -1;
        if (r < P) {
            const unsigned long long *kp = row_keys + (size_t)b * N + r;
            am = key_index(__hip_atomic_load(kp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        }
        s_am[r] = am;
        argmax_out[(size_t)b * N + r] = am;
    }
#pragma unroll
    for (int u = 0; u < kPre; ++u) {
        const int e = u * kAccThreads + tid;
        if (e < N) {
            s_beam[e] = my_beam[u];
            s_slot[e] = min(max(my_slot[u], 0), N - 1);
        }
    }
    if (tid == 0) s_best = -1;
    __syncthreads();                                      // every key has been read
    RD_TR(4);
    for (int r = tid; r < P; r += kAccThreads) row_keys[(size_t)b * N + r] = 0;   // ready for the next call
    if (tid == 0) seq_counters[b] = 0;

    // one thread per candidate (W <= RD_MAX_W <= kAccThreads)
    static_assert(RD_MAX_W <= kAccThreads && RD_MAX_W <= 256, "one thread per candidate, index in 8 bits");
    const int w = tid;
    if (w < W) {
        const int *bm = s_beam + w * L;
        const int *ui = s_slot + w * L;
        int len = 0;
        bool ok = (root_token == nullptr) || (bm[0] == my_root);
        while (ok) {
            ++len;
            if (len == L) break;
            ok = (s_am[ui[len - 1]] == bm[len]);
        }
        n_accept[(size_t)b * W + w] = len;
        // best candidate: longest accepted prefix, smallest index among equals
        atomicMax(&s_best, (len << 8) | (255 - w));
    }
    __syncthreads();
    const int key = s_best;
    const int bl = key >> 8;
    const int bw = 255 - (key & 255);
    const int *bui = s_slot + bw * L;
    for (int t = tid; t < L; t += kAccThreads) accepted_idx[(size_t)b * L + t] = (t < bl) ? bui[t] : -1;
    if (tid == 0) {
        best_beam[b] = bw;
        best_len[b] = bl;
        next_token[b] = (bl > 0) ? s_am[bui[bl - 1]] : my_root;
    }
    RD_TR(5);
}

}  // namespace

extern "C" size_t rd_accept_workspace(int B, int W, int L, int V)
{
    if (rd_check_beam_shape(B, W, L) != RD_OK || V <= 0) return 0;
    return acc_plan(B, W * L, V).total_bytes;
}

// Argument checks shared by the two entry points; *plan is filled on success.
static int accept_check(const float *logits, const int32_t *beams, const int32_t *unpack_index,
                        const int32_t *n_packed, int B, int W, int L, int V,
                        const int32_t *argmax_out, const int32_t *n_accept, const int32_t *best_beam,
                        const int32_t *best_len, const int32_t *next_token, const int32_t *accepted_idx, AccPlan *plan)
{
    const int st = rd_check_beam_shape(B, W, L);
    if (st != RD_OK) return st;
    if (V <= 0) return RD_ERR_INVALID_ARG;
    if (B > 65535) return RD_ERR_UNSUPPORTED;
    if (!logits || !beams || !unpack_index || !n_packed || !argmax_out || !n_accept || !best_beam ||
        !best_len || !next_token || !accepted_idx)
        return RD_ERR_INVALID_ARG;
    if (!rd_aligned(logits, 16)) return RD_ERR_INVALID_ARG;
    *plan = acc_plan(B, W * L, V);
    return RD_OK;
}

// Enqueues the kernel on a zeroed workspace of plan.total_bytes at `ws`.
static int accept_launch(const AccPlan &plan, const float *logits, const int32_t *beams, const int32_t *unpack_index,
                         const int32_t *n_packed, const int32_t *root_token, int B, int W, int L, int V,
                         int32_t *argmax_out, int32_t *n_accept, int32_t *best_beam, int32_t *best_len,
                         int32_t *next_token, int32_t *accepted_idx, unsigned char *ws, hipStream_t stream)
{
    const int N = W * L;
    const dim3 grid(plan.chunks, N, B), block(kAccThreads);
    uint32_t *seq_counters = reinterpret_cast<uint32_t *>(ws);
    uint32_t *row_counters = reinterpret_cast<uint32_t *>(ws + plan.row_counters_off);
    unsigned long long *row_keys = reinterpret_cast<unsigned long long *>(ws + plan.keys_off);
#define RD_ACCEPT_LAUNCH_(U, SPEC)                                                                            \
    hipLaunchKernelGGL((rd_accept_kernel<U, SPEC>), grid, block, 0, stream, logits, beams, unpack_index,       \
                       n_packed, root_token, W, L, V, plan.chunks, plan.chunk_len, argmax_out, n_accept,       \
                       best_beam, best_len, next_token, accepted_idx, seq_counters, row_counters, row_keys)
#define RD_ACCEPT_LAUNCH(U)                                 \
    do {                                                    \
        if (plan.speculate) RD_ACCEPT_LAUNCH_(U, true);     \
        else RD_ACCEPT_LAUNCH_(U, false);                   \
    } while (0)
    switch (plan.loads) {
    case 1: RD_ACCEPT_LAUNCH(1); break;
    case 2: RD_ACCEPT_LAUNCH(2); break;
    case 4: RD_ACCEPT_LAUNCH(4); break;
    case 8: RD_ACCEPT_LAUNCH(8); break;
    case 16: RD_ACCEPT_LAUNCH_(16, false); break;
    default: RD_ACCEPT_LAUNCH_(32, false); break;
    }
#undef RD_ACCEPT_LAUNCH
#undef RD_ACCEPT_LAUNCH_
    return rd_check_launch();
}

extern "C" int rd_accept(const float *logits, const int32_t *beams, const int32_t *unpack_index,
                         const int32_t *n_packed, const int32_t *root_token,
                         int B, int W, int L, int V,
                         int32_t *argmax_out, int32_t *n_accept, int32_t *best_beam,
                         int32_t *best_len, int32_t *next_token, int32_t *accepted_idx,
                         void *workspace, size_t workspace_bytes, void *stream)
{
    AccPlan plan;
    const int st = accept_check(logits, beams, unpack_index, n_packed, B, W, L, V, argmax_out, n_accept, best_beam,
                                best_len, next_token, accepted_idx, &plan);
    if (st != RD_OK) return st;
    if (!workspace || !rd_aligned(workspace, 256) || workspace_bytes < plan.total_bytes) return RD_ERR_WORKSPACE;
    return accept_launch(plan, logits, beams, unpack_index, n_packed, root_token, B, W, L, V, argmax_out, n_accept,
                         best_beam, best_len, next_token, accepted_idx, static_cast<unsigned char *>(workspace),
                         (hipStream_t)stream);
}

// ---- rd_accept_static: the same call for callers that cannot allocate ---------------------------
// The counters and row keys live in a file-scope device array instead of a caller-provided
// workspace.  Every device that loads the library holds its own copy of the array at its own
// address until the process ends; the address is looked up once per device, with that device
// current, and only that address (never the array's name, which in host code is a stand-in and
// not a device address) is handed to kernels.
static __device__ __align__(256) unsigned char scratch[RD_ACCEPT_STATIC_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::atomic<unsigned char *> g_scratch_ptr[kMaxDevices];     // device address of `scratch`, per device, once known

int static_scratch(unsigned char **out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return RD_ERR_HIP;
    if (dev < 0 || dev >= kMaxDevices) return RD_ERR_UNSUPPORTED;
    unsigned char *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p == nullptr) {
        void *sym = nullptr;
        if (hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)) != hipSuccess || sym == nullptr) return RD_ERR_HIP;
        p = static_cast<unsigned char *>(sym);
        g_scratch_ptr[dev].store(p, std::memory_order_release);     // two threads racing here store the same address
    }
    *out = p;
    return RD_OK;
}

// Zeroes n_vec 16-byte vectors.  A kernel rather than a memset so that the call stays safe to
// capture into a HIP graph.
__global__ __launch_bounds__(256) void rd_clear_kernel(uint4 *p, size_t n_vec)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n_vec) p[i] = make_uint4(0, 0, 0, 0);
}

}  // namespace

extern "C" int rd_accept_static(const float *logits, const int32_t *beams, const int32_t *unpack_index,
                                const int32_t *n_packed, const int32_t *root_token,
                                int B, int W, int L, int V,
                                int32_t *argmax_out, int32_t *n_accept, int32_t *best_beam,
                                int32_t *best_len, int32_t *next_token, int32_t *accepted_idx, void *stream)
{
    AccPlan plan;
    const int st = accept_check(logits, beams, unpack_index, n_packed, B, W, L, V, argmax_out, n_accept, best_beam,
                                best_len, next_token, accepted_idx, &plan);
    if (st != RD_OK) return st;
    if (plan.total_bytes > (size_t)RD_ACCEPT_STATIC_BYTES) return RD_ERR_SCRATCH_LIMIT;
    unsigned char *ws = nullptr;
    const int sp = static_scratch(&ws);
    if (sp != RD_OK) return sp;
    // The array keeps whatever the last call on this device left (normally zeros, but a call that was
    // aborted, or one of another shape that failed, may leave anything): clear the part this call uses.
    const size_t n_vec = plan.total_bytes / 16;                     // every section is a multiple of 256 bytes
    hipLaunchKernelGGL(rd_clear_kernel, dim3((unsigned)((n_vec + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
                       reinterpret_cast<uint4 *>(ws), n_vec);
    const int cl = rd_check_launch();
    if (cl != RD_OK) return cl;
    return accept_launch(plan, logits, beams, unpack_index, n_packed, root_token, B, W, L, V, argmax_out, n_accept,
                         best_beam, best_len, next_token, accepted_idx, ws, (hipStream_t)stream);
}
