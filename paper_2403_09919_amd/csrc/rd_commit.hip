// rd_commit: the accepted tokens join the context (Sec. 3.4).  Pure data movement: for each
// (sequence, head) the K and V rows of the accepted packed slots are appended to the cache
// behind ctx_len; one more workgroup per sequence writes the new context length and picks
// the hidden state of the last accepted token.  A few KB per sequence, so the launch is
// latency-bound: every thread issues its 16-byte copy at once, nothing waits on anything else.
#include "rd_internal.h"

namespace {

constexpr int kCommitThreads = 256;

__device__ __forceinline__ int clamp_i(int x, int lo, int hi) { return x < lo ? lo : (x > hi ? hi : x); }

// grid = (H + 1, B): block x < H copies the rows of head x, block x == H does the per-sequence part.
__global__ __launch_bounds__(kCommitThreads) void rd_commit_kernel(
    const uint4 *__restrict__ k_new, const uint4 *__restrict__ v_new,
    const int32_t *__restrict__ accepted_idx, const int32_t *__restrict__ best_len,
    const int32_t *__restrict__ ctx_len, int H, int N, int Cmax, int L, int row_vecs /* 16-byte vectors per K/V row */,
    uint4 *__restrict__ k_cache, uint4 *__restrict__ v_cache, int32_t *__restrict__ ctx_len_out,
    int32_t *__restrict__ n_committed, const uint4 *__restrict__ hidden, int hid_vecs, uint4 *__restrict__ hidden_last,
    const int32_t *__restrict__ block_table /* NULL: dense cache */, int page_size, int max_pages, int n_pages)
{
    const int b = blockIdx.y, h = blockIdx.x, tid = threadIdx.x;
    const int bl = clamp_i(best_len[b], 0, L);
    const int c = clamp_i(ctx_len[b], 0, Cmax);
    const int n = min(bl, Cmax - c);
    if (h == H) {
        if (tid == 0) {
            ctx_len_out[b] = c + n;
            if (n_committed) n_committed[b] = n;
        }
        if (hidden != nullptr && bl > 0) {
            const int slot = clamp_i(accepted_idx[(size_t)b * L + bl - 1], 0, N - 1);
            const uint4 *src = hidden + ((size_t)b * N + slot) * hid_vecs;
            uint4 *dst = hidden_last + (size_t)b * hid_vecs;
            for (int i = tid; i < hid_vecs; i += kCommitThreads) dst[i] = src[i];
        }
        return;
    }
    const size_t bh = (size_t)b * H + h;
    const int total = n * row_vecs;                 // vectors per tensor for this head
    for (int i = tid; i < total; i += kCommitThreads) {
        const int t = i / row_vecs, v = i - t * row_vecs;
        const int slot = clamp_i(accepted_idx[(size_t)b * L + t], 0, N - 1);
        const size_t src = (bh * N + slot) * row_vecs + v;
        size_t dst;
        if (block_table == nullptr) {
            dst = (bh * Cmax + (size_t)(c + t)) * row_vecs + v;
        } else {                                    // position c+t lives in page block_table[b][(c+t)/page_size]
            const int pos = c + t;
            const int page = clamp_i(block_table[(size_t)b * max_pages + pos / page_size], 0, n_pages - 1);
            dst = (((size_t)page * H + h) * page_size + (size_t)(pos % page_size)) * row_vecs + v;
        }
        k_cache[dst] = k_new[src];
        v_cache[dst] = v_new[src];
    }
}

}  // namespace

extern "C" int rd_commit(const void *k_new, const void *v_new, const int32_t *accepted_idx,
                         const int32_t *best_len, const int32_t *ctx_len,
                         int B, int H, int N, int D, int Cmax, int L, rd_dtype dt,
                         void *k_cache, void *v_cache, int32_t *ctx_len_out, int32_t *n_committed,
                         const void *hidden, int Dh, void *hidden_last, void *stream)
{
    if (B <= 0 || H <= 0 || N <= 0 || L <= 0 || Cmax <= 0 || Dh < 0) return RD_ERR_INVALID_ARG;
    if (dt != RD_F32 && dt != RD_BF16 && dt != RD_F16) return RD_ERR_UNSUPPORTED;
    if ((D != 64 && D != 128) || N > RD_MAX_N || L > RD_MAX_N || B > 65535) return RD_ERR_UNSUPPORTED;
    if (!k_new || !v_new || !accepted_idx || !best_len || !ctx_len || !k_cache || !v_cache || !ctx_len_out)
        return RD_ERR_INVALID_ARG;
    if (ctx_len_out == ctx_len) return RD_ERR_INVALID_ARG;
    if (!rd_aligned(k_new, 16) || !rd_aligned(v_new, 16) || !rd_aligned(k_cache, 16) || !rd_aligned(v_cache, 16))
        return RD_ERR_INVALID_ARG;
    const size_t es = dt == RD_F32 ? 4 : 2;
    int hid_vecs = 0;
    if (hidden || hidden_last || Dh) {
        if (!hidden || !hidden_last || Dh <= 0 || (Dh * es) % 16 != 0) return RD_ERR_INVALID_ARG;
        if (!rd_aligned(hidden, 16) || !rd_aligned(hidden_last, 16)) return RD_ERR_INVALID_ARG;
        hid_vecs = (int)(Dh * es / 16);
    }
    const int row_vecs = (int)(D * es / 16);
    hipLaunchKernelGGL(rd_commit_kernel, dim3(H + 1, B), dim3(kCommitThreads), 0, (hipStream_t)stream,
                       static_cast<const uint4 *>(k_new), static_cast<const uint4 *>(v_new), accepted_idx, best_len,
                       ctx_len, H, N, Cmax, L, row_vecs, static_cast<uint4 *>(k_cache), static_cast<uint4 *>(v_cache),
                       ctx_len_out, n_committed, static_cast<const uint4 *>(hidden), hid_vecs,
                       static_cast<uint4 *>(hidden_last), nullptr, 0, 0, 0);
    return rd_check_launch();
}

extern "C" int rd_commit_paged(const void *k_new, const void *v_new, const int32_t *accepted_idx,
                               const int32_t *best_len, const int32_t *ctx_len,
                               int B, int H, int N, int D, int L, rd_dtype dt,
                               void *k_pages, void *v_pages, const int32_t *block_table,
                               int page_size, int max_pages, int n_pages,
                               int32_t *ctx_len_out, int32_t *n_committed,
                               const void *hidden, int Dh, void *hidden_last, void *stream)
{
    if (B <= 0 || H <= 0 || N <= 0 || L <= 0 || page_size <= 0 || max_pages <= 0 || n_pages <= 0 || Dh < 0)
        return RD_ERR_INVALID_ARG;
    if (dt != RD_F32 && dt != RD_BF16 && dt != RD_F16) return RD_ERR_UNSUPPORTED;
    if ((D != 64 && D != 128) || N > RD_MAX_N || L > RD_MAX_N || B > 65535) return RD_ERR_UNSUPPORTED;
    if ((long long)page_size * max_pages > (1ll << 30)) return RD_ERR_UNSUPPORTED;
    if (!k_new || !v_new || !accepted_idx || !best_len || !ctx_len || !k_pages || !v_pages || !block_table || !ctx_len_out)
        return RD_ERR_INVALID_ARG;
    if (ctx_len_out == ctx_len) return RD_ERR_INVALID_ARG;
    if (!rd_aligned(k_new, 16) || !rd_aligned(v_new, 16) || !rd_aligned(k_pages, 16) || !rd_aligned(v_pages, 16) ||
        !rd_aligned(block_table, 4))
        return RD_ERR_INVALID_ARG;
    const size_t es = dt == RD_F32 ? 4 : 2;
    int hid_vecs = 0;
    if (hidden || hidden_last || Dh) {
        if (!hidden || !hidden_last || Dh <= 0 || (Dh * es) % 16 != 0) return RD_ERR_INVALID_ARG;
        if (!rd_aligned(hidden, 16) || !rd_aligned(hidden_last, 16)) return RD_ERR_INVALID_ARG;
        hid_vecs = (int)(Dh * es / 16);
    }
    const int row_vecs = (int)(D * es / 16);
    hipLaunchKernelGGL(rd_commit_kernel, dim3(H + 1, B), dim3(kCommitThreads), 0, (hipStream_t)stream,
                       static_cast<const uint4 *>(k_new), static_cast<const uint4 *>(v_new), accepted_idx, best_len,
                       ctx_len, H, N, page_size * max_pages, L, row_vecs, static_cast<uint4 *>(k_pages),
                       static_cast<uint4 *>(v_pages), ctx_len_out, n_committed, static_cast<const uint4 *>(hidden),
                       hid_vecs, static_cast<uint4 *>(hidden_last), block_table, page_size, max_pages, n_pages);
    return rd_check_launch();
}
