// rd_dedup: dynamic tree attention construction (Sec. 3.3, App. A.1) for gfx950.
//
// One workgroup per sequence, everything in LDS, data-parallel phases separated by barriers
// (the whole input is a few hundred bytes; what costs time is dependent latency, so no phase
// is a serial walk over positions):
//   A  stage the W x L candidates; owner[i][j] = i.
//   B  one thread per ordered pair (i, k < i): walk their common prefix and lower owner[i][j]
//      to k (LDS atomic min) for every j inside it.  Afterwards owner[i][j] is the smallest
//      candidate sharing i's first j+1 tokens, i.e. prefix_tree — the equal-length property
//      the paper exploits, with no trie and no data-dependent pointer chasing.
//   C  a token is kept iff owner == i; kept tokens of a candidate are a suffix of its row, so
//      each row's first kept position and a prefix sum of the kept counts give every row
//      its first packed slot (row-major slot order).
//   D  one thread per token: slot of its owner's copy -> unpack_index.
//   E  one thread per kept token: packed token, parent, position id, and the mask row as the
//      OR of the slots on its path.
//   F  paddings, the bit-packed and the dense mask, with coalesced stores.
#include "rd_internal.h"

RD_TRACE_DEFINE(rd_debug_set_trace_dedup)

namespace {

constexpr int kDedupThreads = 384;
constexpr int kMaskWords = (RD_MAX_N + 63) / 64;

__global__ __launch_bounds__(kDedupThreads) void rd_dedup_kernel(
    const int32_t *__restrict__ beams, const int32_t *__restrict__ ctx_len, int W, int L,
    int32_t *__restrict__ prefix_tree, int32_t *__restrict__ packed_tokens,
    int32_t *__restrict__ n_packed, int32_t *__restrict__ unpack_index,
    int32_t *__restrict__ parent, int32_t *__restrict__ position_ids,
    uint8_t *__restrict__ tree_mask, uint64_t *__restrict__ tree_mask_bits)
{
    __shared__ int32_t s_beam[RD_MAX_N];
    __shared__ int32_t s_owner[RD_MAX_N];          // prefix_tree of this sequence
    __shared__ int32_t s_slot[RD_MAX_N];           // unpack_index of this sequence
    __shared__ int32_t s_base[RD_MAX_W + 1], s_first[RD_MAX_W + 1];
    __shared__ uint64_t s_bits[RD_MAX_N][kMaskWords];   // mask row of each packed slot
    __shared__ int s_P;

    const int b = blockIdx.x;
    const int tid = threadIdx.x;
    const int N = W * L;
    const int words = (N + 63) >> 6;
    const size_t seq = (size_t)b * N;
    RD_TR(0);
    const int ctx = ctx_len ? ctx_len[b] : 0;      // fetched with the candidates, not after them

    // N <= RD_MAX_N <= kDedupThreads: thread e owns token e = (i, j) in every per-token phase.
    static_assert(RD_MAX_N <= kDedupThreads, "one thread per token");
    const int e = tid;
    const bool tok = e < N;
    const int i = tok ? e / L : 0, j = tok ? e - i * L : 0;

    // ---- A: stage -----------------------------------------------------------------------------------
    if (tok) {
        s_beam[e] = beams[seq + e];
        s_owner[e] = i;
#pragma unroll
        for (int w = 0; w < kMaskWords; ++w) s_bits[e][w] = 0;
    }
    if (tid < W) s_first[tid] = L;
    __syncthreads();
    RD_TR(1);

    // ---- B: common prefixes of all pairs ----------------------------------------------------------------
    // Both rows are read eight tokens at a time (independent LDS reads), the match length follows
    // in registers, and the atomics that lower the owners are issued without waiting on each other.
    for (int pr = tid; pr < W * W; pr += kDedupThreads) {
        const int pi = pr / W, pk = pr - pi * W;
        if (pk < pi) {
            const int32_t *ri = s_beam + pi * L, *rk = s_beam + pk * L;
            for (int j0 = 0; j0 < L; j0 += 8) {
                int32_t a[8], c[8];
#pragma unroll
                for (int t = 0; t < 8; ++t) {
                    const int jj = min(j0 + t, L - 1);
                    a[t] = ri[jj];
                    c[t] = rk[jj];
                }
                int m = 0;                          // matching tokens at the head of this group
                bool run = true;
#pragma unroll
                for (int t = 0; t < 8; ++t) {
                    run = run && (j0 + t < L) && (a[t] == c[t]);
                    m += run ? 1 : 0;
                }
#pragma unroll
                for (int t = 0; t < 8; ++t)
                    if (t < m) atomicMin(&s_owner[pi * L + j0 + t], pk);
                if (m < 8) break;
            }
        }
    }
    rd_lds_barrier();
    RD_TR(2);

    // ---- C: first kept position per row (kept tokens are a suffix of their row) ---------------------------
    const int owner = tok ? s_owner[e] : 0;        // prefix_tree[i][j]
    if (tok && owner == i) atomicMin(&s_first[i], j);
    rd_lds_barrier();
    // exclusive prefix sum of the kept counts = first packed slot of each row (row-major slot order)
    if (tid <= W) {                                 // thread W computes the total
        int base = 0;
        for (int k = 0; k < tid; ++k) base += L - s_first[k];
        if (tid < W) s_base[tid] = base;
        else { s_P = base; n_packed[b] = base; }
    }
    rd_lds_barrier();
    RD_TR(3);

    // ---- D: one thread per token: slot of its owner's copy -> unpack_index -----------------------------------
    if (tok) {
        const int slot = s_base[owner] + j - s_first[owner];   // (owner, j) is a kept token: j >= first_kept[owner]
        s_slot[e] = slot;
        unpack_index[seq + e] = slot;
        if (prefix_tree) prefix_tree[seq + e] = owner;
    }
    rd_lds_barrier();

    // ---- E: one thread per kept token ---------------------------------------------------------------------------
    if (tok && owner == i) {
        const int slot = s_slot[e];
        packed_tokens[seq + slot] = s_beam[e];
        parent[seq + slot] = j ? s_slot[e - 1] : -1;
        position_ids[seq + slot] = ctx + j;
        uint64_t path[kMaskWords];             // slots on the path from the root to (i, j)
#pragma unroll
        for (int w = 0; w < kMaskWords; ++w) path[w] = 0;
        for (int t = 0; t <= j; ++t) {
            const int q = s_slot[i * L + t];
#pragma unroll
            for (int w = 0; w < kMaskWords; ++w)
                if ((q >> 6) == w) path[w] |= 1ull << (q & 63);
        }
#pragma unroll
        for (int w = 0; w < kMaskWords; ++w) s_bits[slot][w] = path[w];
    }
    rd_lds_barrier();
    RD_TR(4);

    // ---- F: paddings and masks ---------------------------------------------------------------------------------
    const int P = s_P;
    for (int p = P + tid; p < N; p += kDedupThreads) {
        packed_tokens[seq + p] = -1;
        parent[seq + p] = -1;
        position_ids[seq + p] = -1;
    }
    if (tree_mask_bits) {
        uint64_t *dst = tree_mask_bits + seq * words;
        for (int i = tid; i < N * words; i += kDedupThreads) dst[i] = s_bits[i / words][i % words];
    }
    if (tree_mask) {
        uint8_t *dst = tree_mask + seq * N;
        if ((N & 3) == 0) {                          // N*N and seq*N are multiples of 4: 32-bit stores
            uint32_t *dst4 = reinterpret_cast<uint32_t *>(dst);
            const int n4 = N >> 2;
            for (int i = tid; i < N * n4; i += kDedupThreads) {
                const int p = i / n4, q0 = (i % n4) << 2;
                const uint64_t w = s_bits[p][q0 >> 6] >> (q0 & 63);
                dst4[i] = (uint32_t)(w & 1) | (uint32_t)((w >> 1) & 1) << 8 |
                          (uint32_t)((w >> 2) & 1) << 16 | (uint32_t)((w >> 3) & 1) << 24;
            }
        } else {
            for (int i = tid; i < N * N; i += kDedupThreads) {
                const int p = i / N, q = i % N;
                dst[i] = (uint8_t)((s_bits[p][q >> 6] >> (q & 63)) & 1);
            }
        }
    }
    RD_TR(5);
}

}  // namespace

extern "C" int rd_dedup(const int32_t *beams, const int32_t *ctx_len, int B, int W, int L,
                        int32_t *prefix_tree, int32_t *packed_tokens, int32_t *n_packed,
                        int32_t *unpack_index, int32_t *parent, int32_t *position_ids,
                        uint8_t *tree_mask, uint64_t *tree_mask_bits, void *stream)
{
    const int st = rd_check_beam_shape(B, W, L);
    if (st != RD_OK) return st;
    if (!beams || !packed_tokens || !n_packed || !unpack_index || !parent || !position_ids)
        return RD_ERR_INVALID_ARG;
    if (!rd_aligned(tree_mask, 4) || !rd_aligned(tree_mask_bits, 8)) return RD_ERR_INVALID_ARG;
    hipLaunchKernelGGL(rd_dedup_kernel, dim3(B), dim3(kDedupThreads), 0, (hipStream_t)stream,
                       beams, ctx_len, W, L, prefix_tree, packed_tokens, n_packed, unpack_index,
                       parent, position_ids, tree_mask, tree_mask_bits);
    return rd_check_launch();
}
