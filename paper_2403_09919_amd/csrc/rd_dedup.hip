// rd_dedup: dynamic tree attention construction (Sec. 3.3, App. A.1) for gfx950.
//
// One workgroup per sequence.  Wave 0 does the whole prefix analysis with lane i
// owning candidate i (W <= 64):
//   * the lane keeps a 64-bit set `alive` of the candidates whose prefix so far
//     equals its own; at position j it is intersected with the ballot of lanes
//     holding the same token.  prefix_tree[i][j] is the lowest set bit.  This is the
//     equal-length property the paper exploits: no trie, no data-dependent walks.
//   * a token is kept iff its lane is that lowest bit; kept tokens of a lane are a
//     suffix of its row, so a lane's kept count is L - first_kept and one wave
//     exclusive scan gives every lane its first packed slot (row-major slot order).
//   * a second sweep over j turns (owner, j) into slots and carries the ancestor
//     bit set along the row, which is the tree-mask row of every kept token.
// The mask rows are staged in LDS; all four waves then write the dense and the
// bit-packed masks and the paddings with coalesced stores.
#include "rd_internal.h"

namespace {

constexpr int kDedupThreads = 256;

__device__ __forceinline__ int wave_excl_scan(int v, int lane, int *total)
{
    int incl = v;
#pragma unroll
    for (int off = 1; off < RD_WAVE; off <<= 1) {
        const int up = __shfl_up(incl, off, RD_WAVE);
        if (lane >= off) incl += up;
    }
    *total = __shfl(incl, RD_WAVE - 1, RD_WAVE);
    return incl - v;
}

__global__ __launch_bounds__(kDedupThreads) void rd_dedup_kernel(
    const int32_t *__restrict__ beams, const int32_t *__restrict__ ctx_len, int W, int L,
    int32_t *__restrict__ prefix_tree, int32_t *__restrict__ packed_tokens,
    int32_t *__restrict__ n_packed, int32_t *__restrict__ unpack_index,
    int32_t *__restrict__ parent, int32_t *__restrict__ position_ids,
    uint8_t *__restrict__ tree_mask, uint64_t *__restrict__ tree_mask_bits)
{
    __shared__ int32_t s_beam[RD_MAX_N];
    __shared__ int32_t s_owner[RD_MAX_N];          // prefix_tree of this sequence
    __shared__ uint64_t s_bits[RD_MAX_N][2];       // mask row of each packed slot
    __shared__ int s_P;

    const int b = blockIdx.x;
    const int tid = threadIdx.x;
    const int N = W * L;
    const int words = (N + 63) >> 6;
    const size_t seq = (size_t)b * N;
    const int ctx = ctx_len ? ctx_len[b] : 0;      // fetched with the candidates, not after them

    for (int i = tid; i < N; i += kDedupThreads) {
        s_beam[i] = beams[seq + i];
        s_bits[i][0] = 0;
        s_bits[i][1] = 0;
    }
    __syncthreads();

    if (tid < RD_WAVE) {
        const int lane = tid;
        const bool active = lane < W;
        const int row = active ? lane : 0;          // idle lanes shadow candidate 0, write nothing

        uint64_t alive = (W == 64) ? ~0ull : ((1ull << W) - 1ull);
        int first_kept = L;
        for (int j = 0; j < L; ++j) {
            const int tok = s_beam[row * L + j];
            uint64_t same = 0;
            for (int k = 0; k < W; ++k) {
                const int tk = __builtin_amdgcn_readlane(tok, k);               // candidate k's token (k is uniform)
                const uint64_t eq = __builtin_amdgcn_ballot_w64(tok == tk);     // lanes whose token equals it
                same = (lane == k) ? eq : same;
            }
            alive &= same;
            const int owner = __ffsll((unsigned long long)alive) - 1;   // >= 0: the lane itself is in alive
            if (active) {
                s_owner[lane * L + j] = owner;
                if (owner == lane && first_kept == L) first_kept = j;
            }
        }
        int P;
        const int base = wave_excl_scan(active ? L - first_kept : 0, lane, &P);
        if (lane == 0) { s_P = P; n_packed[b] = P; }

        uint64_t anc0 = 0, anc1 = 0;                // slots on the path from the root to (lane, j)
        int prev = -1;
        for (int j = 0; j < L; ++j) {
            const int owner = active ? s_owner[lane * L + j] : 0;
            // (owner, j) is a kept token: j >= first_kept[owner]
            const int slot = __shfl(base, owner, RD_WAVE) + j - __shfl(first_kept, owner, RD_WAVE);
            if (slot < 64) anc0 |= 1ull << slot; else anc1 |= 1ull << (slot - 64);
            if (active) {
                unpack_index[seq + lane * L + j] = slot;
                if (prefix_tree) prefix_tree[seq + lane * L + j] = owner;
                if (owner == lane) {
                    packed_tokens[seq + slot] = s_beam[lane * L + j];
                    parent[seq + slot] = prev;
                    position_ids[seq + slot] = ctx + j;
                    s_bits[slot][0] = anc0;
                    s_bits[slot][1] = anc1;
                }
            }
            prev = slot;
        }
    }
    __syncthreads();

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
