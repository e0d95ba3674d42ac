// rd_tree_attn host entry: argument checks, split plan, dispatch to the MFMA kernel (bf16 or
// fp16 elements) or the fp32 kernel.  See rd_attn_common.h for the decomposition.
#include "rd_attn_common.h"

namespace rd {
int tree_attn_bf16(const AttnArgs &a, int D, int waves, int rg_tiles, hipStream_t stream);
int tree_attn_f16(const AttnArgs &a, int D, int waves, int rg_tiles, hipStream_t stream);
int tree_attn_paged(const AttnArgs &a, int D, int waves, int rg_tiles, bool f16, hipStream_t stream);
int tree_attn_f32(const AttnArgs &a, int D, hipStream_t stream);
int tree_attn_rope_bf16(const AttnArgs &a, int D, int waves, int rg_tiles, hipStream_t stream);
int tree_attn_rope_f16(const AttnArgs &a, int D, int waves, int rg_tiles, hipStream_t stream);
}  // namespace rd

static int attn_check_shape(int B, int H, int N, int D, int Cmax, rd_dtype dt)
{
    if (B <= 0 || H <= 0 || N <= 0 || D <= 0 || Cmax < 0) return RD_ERR_INVALID_ARG;
    if (dt != RD_F32 && dt != RD_BF16 && dt != RD_F16) return RD_ERR_UNSUPPORTED;
    if (N > RD_MAX_N) return RD_ERR_UNSUPPORTED;
    if (D != 64 && D != 128) return RD_ERR_UNSUPPORTED;
    if ((long long)B * H > (1ll << 24)) return RD_ERR_UNSUPPORTED;
    return RD_OK;
}

extern "C" size_t rd_tree_attn_workspace(int B, int H, int N, int D, int Cmax, rd_dtype dt)
{
    if (attn_check_shape(B, H, N, D, Cmax, dt) != RD_OK) return 0;
    return rd::attn_plan(B, H, N, D, Cmax, dt == RD_F32 ? 4 : 2).total_bytes;
}

// Dense entry points: `plan_ctx` is the context length the launch plan is made for (the cache's
// capacity Cmax, or a caller-supplied bound on the live contexts); the kernels themselves take every
// sequence's range from its own ctx_len, whatever the plan assumed.
static int tree_attn_dense(const void *q, const void *k_cache, const void *v_cache,
                           const int32_t *ctx_len, const void *k_new, const void *v_new,
                           const int32_t *n_packed, const uint64_t *tree_mask_bits,
                           int B, int H, int N, int D, int Cmax, int plan_ctx, rd_dtype dt, float scale,
                           void *out, void *workspace, size_t workspace_bytes, void *stream)
{
    const int st = attn_check_shape(B, H, N, D, Cmax, dt);
    if (st != RD_OK) return st;
    if (!q || !k_new || !v_new || !ctx_len || !n_packed || !tree_mask_bits || !out) return RD_ERR_INVALID_ARG;
    if (Cmax > 0 && (!k_cache || !v_cache)) return RD_ERR_INVALID_ARG;
    if (!rd_aligned(q, 16) || !rd_aligned(k_cache, 16) || !rd_aligned(v_cache, 16) || !rd_aligned(k_new, 16) ||
        !rd_aligned(v_new, 16) || !rd_aligned(out, 16) || !rd_aligned(tree_mask_bits, 8))
        return RD_ERR_INVALID_ARG;
    const rd::AttnPlan plan = rd::attn_plan(B, H, N, D, plan_ctx, dt == RD_F32 ? 4 : 2);
    if (!workspace || !rd_aligned(workspace, 256) || workspace_bytes < plan.total_bytes) return RD_ERR_WORKSPACE;

    rd::AttnArgs a;
    a.q = q; a.k_cache = k_cache; a.v_cache = v_cache; a.k_new = k_new; a.v_new = v_new;
    a.ctx_len = ctx_len; a.n_packed = n_packed; a.mask_bits = tree_mask_bits; a.out = out;
    a.counters = static_cast<unsigned long long *>(workspace);
    a.partials = reinterpret_cast<float *>(static_cast<unsigned char *>(workspace) + plan.counters_bytes);
    a.B = B; a.H = H; a.N = N; a.Cmax = Cmax; a.S = plan.S; a.words = (N + 63) / 64; a.rows_pad = plan.rows_pad;
    a.scale_log2e = scale * 1.44269504088896340736f;
    a.xcd_remap = (((long long)B * H) % 8 == 0) ? 1 : 0;
    a.fuse_tree = plan.fuse_tree;
    a.n_rg = plan.n_rg;
    a.block_table = nullptr; a.page_size = 0; a.max_pages = 0; a.n_pages = 0;
    a.position_ids = nullptr; a.cos_tab = nullptr; a.sin_tab = nullptr; a.max_pos = 0; a.k_rot = nullptr;
    if (dt == RD_BF16) return rd::tree_attn_bf16(a, D, plan.waves, plan.rg_tiles, (hipStream_t)stream);
    if (dt == RD_F16) return rd::tree_attn_f16(a, D, plan.waves, plan.rg_tiles, (hipStream_t)stream);
    return rd::tree_attn_f32(a, D, (hipStream_t)stream);
}

extern "C" int rd_tree_attn(const void *q, const void *k_cache, const void *v_cache,
                            const int32_t *ctx_len, const void *k_new, const void *v_new,
                            const int32_t *n_packed, const uint64_t *tree_mask_bits,
                            int B, int H, int N, int D, int Cmax, rd_dtype dt, float scale,
                            void *out, void *workspace, size_t workspace_bytes, void *stream)
{
    return tree_attn_dense(q, k_cache, v_cache, ctx_len, k_new, v_new, n_packed, tree_mask_bits, B, H, N, D, Cmax, Cmax, dt,
                           scale, out, workspace, workspace_bytes, stream);
}

extern "C" int rd_tree_attn_bounded(const void *q, const void *k_cache, const void *v_cache,
                                    const int32_t *ctx_len, const void *k_new, const void *v_new,
                                    const int32_t *n_packed, const uint64_t *tree_mask_bits,
                                    int B, int H, int N, int D, int Cmax, int ctx_bound, rd_dtype dt, float scale,
                                    void *out, void *workspace, size_t workspace_bytes, void *stream)
{
    if (ctx_bound < 0) return RD_ERR_INVALID_ARG;
    return tree_attn_dense(q, k_cache, v_cache, ctx_len, k_new, v_new, n_packed, tree_mask_bits, B, H, N, D, Cmax,
                           ctx_bound < Cmax ? ctx_bound : Cmax, dt, scale, out, workspace, workspace_bytes, stream);
}

// ---- paged KV cache ---------------------------------------------------------------------------
static int paged_check_shape(int B, int H, int N, int D, int page_size, int max_pages, int n_pages, rd_dtype dt)
{
    if (page_size <= 0 || max_pages <= 0 || n_pages <= 0) return RD_ERR_INVALID_ARG;
    if (dt != RD_BF16 && dt != RD_F16) return RD_ERR_UNSUPPORTED;            // 16-bit caches only
    if (page_size % 32 != 0) return RD_ERR_UNSUPPORTED;                      // a 32-key tile must not straddle pages
    if ((long long)page_size * max_pages > (1ll << 30)) return RD_ERR_UNSUPPORTED;
    return attn_check_shape(B, H, N, D, page_size * max_pages, dt);
}

extern "C" size_t rd_tree_attn_paged_workspace(int B, int H, int N, int D, int page_size, int max_pages, rd_dtype dt)
{
    if (paged_check_shape(B, H, N, D, page_size, max_pages, 1, dt) != RD_OK) return 0;
    return rd::attn_plan(B, H, N, D, page_size * max_pages, 2).total_bytes;
}

extern "C" int rd_tree_attn_paged(const void *q, const void *k_pages, const void *v_pages,
                                  const int32_t *block_table, int page_size, int max_pages, int n_pages,
                                  const int32_t *ctx_len, const void *k_new, const void *v_new,
                                  const int32_t *n_packed, const uint64_t *tree_mask_bits,
                                  int B, int H, int N, int D, rd_dtype dt, float scale,
                                  void *out, void *workspace, size_t workspace_bytes, void *stream)
{
    const int st = paged_check_shape(B, H, N, D, page_size, max_pages, n_pages, dt);
    if (st != RD_OK) return st;
    if (!q || !k_pages || !v_pages || !block_table || !k_new || !v_new || !ctx_len || !n_packed || !tree_mask_bits || !out)
        return RD_ERR_INVALID_ARG;
    if (!rd_aligned(q, 16) || !rd_aligned(k_pages, 16) || !rd_aligned(v_pages, 16) || !rd_aligned(k_new, 16) ||
        !rd_aligned(v_new, 16) || !rd_aligned(out, 16) || !rd_aligned(tree_mask_bits, 8) || !rd_aligned(block_table, 4))
        return RD_ERR_INVALID_ARG;
    const int Cmax = page_size * max_pages;
    const rd::AttnPlan plan = rd::attn_plan(B, H, N, D, Cmax, 2);
    if (!workspace || !rd_aligned(workspace, 256) || workspace_bytes < plan.total_bytes) return RD_ERR_WORKSPACE;

    rd::AttnArgs a;
    a.q = q; a.k_cache = k_pages; a.v_cache = v_pages; a.k_new = k_new; a.v_new = v_new;
    a.ctx_len = ctx_len; a.n_packed = n_packed; a.mask_bits = tree_mask_bits; a.out = out;
    a.block_table = block_table; a.page_size = page_size; a.max_pages = max_pages; a.n_pages = n_pages;
    a.counters = static_cast<unsigned long long *>(workspace);
    a.partials = reinterpret_cast<float *>(static_cast<unsigned char *>(workspace) + plan.counters_bytes);
    a.B = B; a.H = H; a.N = N; a.Cmax = Cmax; a.S = plan.S; a.words = (N + 63) / 64; a.rows_pad = plan.rows_pad;
    a.scale_log2e = scale * 1.44269504088896340736f;
    a.xcd_remap = (((long long)B * H) % 8 == 0) ? 1 : 0;
    a.fuse_tree = plan.fuse_tree;
    a.n_rg = plan.n_rg;
    a.position_ids = nullptr; a.cos_tab = nullptr; a.sin_tab = nullptr; a.max_pos = 0; a.k_rot = nullptr;
    return rd::tree_attn_paged(a, D, plan.waves, plan.rg_tiles, dt == RD_F16, (hipStream_t)stream);
}

// ---- rotary embedding fused into the call -------------------------------------------------------
extern "C" int rd_tree_attn_rope(const void *q, const void *k_cache, const void *v_cache,
                                 const int32_t *ctx_len, const void *k_new, const void *v_new,
                                 const int32_t *n_packed, const uint64_t *tree_mask_bits,
                                 const int32_t *position_ids, const float *cos_tab, const float *sin_tab, int max_pos,
                                 int B, int H, int N, int D, int Cmax, rd_dtype dt, float scale,
                                 void *out, void *k_new_rot, void *workspace, size_t workspace_bytes, void *stream)
{
    const int st = attn_check_shape(B, H, N, D, Cmax, dt);
    if (st != RD_OK) return st;
    if (dt != RD_BF16 && dt != RD_F16) return RD_ERR_UNSUPPORTED;            // the matrix-core kernels only
    if (max_pos <= 0) return RD_ERR_INVALID_ARG;
    if (!q || !k_new || !v_new || !ctx_len || !n_packed || !tree_mask_bits || !out || !position_ids || !cos_tab || !sin_tab)
        return RD_ERR_INVALID_ARG;
    if (Cmax > 0 && (!k_cache || !v_cache)) return RD_ERR_INVALID_ARG;
    if (!rd_aligned(q, 16) || !rd_aligned(k_cache, 16) || !rd_aligned(v_cache, 16) || !rd_aligned(k_new, 16) ||
        !rd_aligned(v_new, 16) || !rd_aligned(out, 16) || !rd_aligned(k_new_rot, 16) || !rd_aligned(tree_mask_bits, 8) ||
        !rd_aligned(cos_tab, 4) || !rd_aligned(sin_tab, 4) || !rd_aligned(position_ids, 4))
        return RD_ERR_INVALID_ARG;
    if (k_new_rot == k_new || k_new_rot == q) return RD_ERR_INVALID_ARG;    // other workgroups still read the unrotated rows
    const rd::AttnPlan plan = rd::attn_plan(B, H, N, D, Cmax, 2);
    if (!workspace || !rd_aligned(workspace, 256) || workspace_bytes < plan.total_bytes) return RD_ERR_WORKSPACE;

    rd::AttnArgs a;
    a.q = q; a.k_cache = k_cache; a.v_cache = v_cache; a.k_new = k_new; a.v_new = v_new;
    a.ctx_len = ctx_len; a.n_packed = n_packed; a.mask_bits = tree_mask_bits; a.out = out;
    a.counters = static_cast<unsigned long long *>(workspace);
    a.partials = reinterpret_cast<float *>(static_cast<unsigned char *>(workspace) + plan.counters_bytes);
    a.B = B; a.H = H; a.N = N; a.Cmax = Cmax; a.S = plan.S; a.words = (N + 63) / 64; a.rows_pad = plan.rows_pad;
    a.scale_log2e = scale * 1.44269504088896340736f;
    a.xcd_remap = (((long long)B * H) % 8 == 0) ? 1 : 0;
    a.fuse_tree = plan.fuse_tree;
    a.n_rg = plan.n_rg;
    a.block_table = nullptr; a.page_size = 0; a.max_pages = 0; a.n_pages = 0;
    a.position_ids = position_ids; a.cos_tab = cos_tab; a.sin_tab = sin_tab; a.max_pos = max_pos; a.k_rot = k_new_rot;
    if (dt == RD_BF16) return rd::tree_attn_rope_bf16(a, D, plan.waves, plan.rg_tiles, (hipStream_t)stream);
    return rd::tree_attn_rope_f16(a, D, plan.waves, plan.rg_tiles, (hipStream_t)stream);
}
