/*
 * rd.h — C ABI of the ReDrafter verification step on AMD MI355X (gfx950).
 *
 * One speculative-decoding step of ReDrafter (arXiv 2403.09919, Sec. 3.4) verifies the
 * drafter's beam with the LLM.  This library implements the parts of that step that are
 * not the LLM's dense layers:
 *
 *   rd_dedup      dynamic tree attention construction (Sec. 3.3, App. A.1): remove the
 *                 duplicated prefixes of W candidates of length L, giving a packed token
 *                 set plus the tree mask, parents, position ids and the unpack index;
 *   rd_tree_attn  the attention core of the LLM's forward pass over the packed tokens
 *                 with that mask, against the KV cache (Sec. 3.3, 3.4);
 *   rd_accept     greedy "token match" acceptance (Sec. 3.4, Fig. 2): arg max of the
 *                 LLM's logits per packed token, longest accepted prefix per candidate,
 *                 best candidate, next token;
 *   rd_accept_sample  the same selection by rejection sampling, for sampling at a temperature;
 *   rd_commit     what follows acceptance (Sec. 3.4): the accepted tokens join the context
 *                 (their K/V rows are appended to the cache, ctx_len grows) and the LLM's
 *                 hidden state at the last accepted token is picked out for the next draft;
 *   rd_rope       rotary position embedding of the packed queries and keys at rd_dedup's
 *                 position ids (for LLaMA-family LLMs such as the paper's Vicuna models).
 *   rd_draft      the step before: the draft model and its beam search (Sec. 3.1, 3.2), which
 *                 produce the candidates.
 * rd_tree_attn_paged and rd_commit_paged are the same over a paged KV cache.
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers to dense row-major arrays (last index
 *     fastest).  The caller owns every buffer; the library never allocates, frees or
 *     synchronises.  A call only enqueues kernels on `stream` (a hipStream_t passed as
 *     void*; NULL = the default stream); outputs are valid once the stream reaches
 *     that point.  Calls may be captured into a HIP graph.
 *   - A batch is B independent sequences (App. A.1).  N = W*L is the padded packed
 *     length; sequence b has n_packed[b] <= N packed tokens.
 *   - Return value: RD_OK or a negative rd_status.  Nothing is thrown, printed or
 *     aborted.  Argument errors that the host can see (NULL required pointer,
 *     non-positive or unsupported sizes, unknown dtype, misaligned pointer, workspace
 *     too small) are rejected before anything is launched.  Data preconditions that
 *     live on the device (0 <= ctx_len[b] <= Cmax, n_packed[b] <= N, logits free of
 *     NaN) are not checked; ctx_len and n_packed are clamped into range.
 *   - Limits: 1 <= W <= 128, L >= 1, N = W*L <= 384, D in {64, 128} (the paper's widest beams,
 *     Sec. 4.3: 70 candidates of 5 tokens, are N = 350).
 */
#ifndef RD_H
#define RD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    RD_F32 = 0, RD_BF16 = 1, RD_F16 = 2,
    /* not element types: the two bounds make every int a valid value of the type, so that a wrong code
       passed by a caller is an RD_ERR_UNSUPPORTED return and never undefined behaviour */
    RD_DTYPE_RANGE_LO = -2147483647 - 1, RD_DTYPE_RANGE_HI = 2147483647
} rd_dtype;

typedef enum {
    RD_OK = 0,
    RD_ERR_INVALID_ARG = -1, /* NULL required pointer, size <= 0, bad alignment */
    RD_ERR_UNSUPPORTED = -2, /* size or dtype outside the limits above */
    RD_ERR_WORKSPACE = -3,   /* workspace NULL or smaller than rd_*_workspace() */
    RD_ERR_HIP = -4,         /* a kernel launch failed (hipGetLastError) */
    RD_ERR_SCRATCH_LIMIT = -5 /* rd_accept_static: the sizes need more than the library's static scratch array */
} rd_status;

#define RD_MAX_W 128
#define RD_MAX_N 384

/* Static description of a status code; never NULL. */
const char *rd_strerror(int code);

/* Library version: major*10000 + minor*100 + patch. */
int rd_version(void);

/*
 * rd_dedup — dedup_prefix + pack_beam + tree structure (Sec. 3.3, App. A.1).
 *
 *   prefix_tree[b][i][j]  smallest candidate index k whose first j+1 tokens equal
 *                         candidate i's (the App. A.1 definition).
 *   A token (i,j) is kept iff prefix_tree[b][i][j] == i ("condense tokens where
 *   prefix_tree[i][j] < i").  Kept tokens get packed slots 0..n_packed[b]-1 in
 *   row-major (i, j) order.
 *   packed_tokens[b][p]   token at slot p                                 (pad -1)
 *   unpack_index[b][i][j] slot holding candidate i's j-th token
 *   parent[b][p]          slot of the previous token on p's path, -1 at depth 0 (pad -1)
 *   position_ids[b][p]    ctx_len[b] + depth of p; depth alone if ctx_len == NULL (pad -1)
 *   tree_mask[b][p][q]    1 iff q == p or q is an ancestor of p (what p may attend
 *                         to among the packed tokens); pad rows and columns 0
 *   tree_mask_bits[b][p][w] bit (q & 63) of word (q >> 6) = tree_mask[b][p][q]
 *
 * beams: int32 [B,W,L], any token values.  Outputs: int32 [B,W,L] / [B,N] / [B];
 * tree_mask uint8 [B,N,N]; tree_mask_bits uint64 [B,N,ceil(N/64)].  prefix_tree,
 * tree_mask and tree_mask_bits may each be NULL (not written); the others are required.
 */
int rd_dedup(const int32_t *beams, const int32_t *ctx_len, int B, int W, int L,
             int32_t *prefix_tree, int32_t *packed_tokens, int32_t *n_packed,
             int32_t *unpack_index, int32_t *parent, int32_t *position_ids,
             uint8_t *tree_mask, uint64_t *tree_mask_bits, void *stream);

/*
 * rd_tree_attn — tree-masked attention of the packed candidates (Sec. 3.3, 3.4).
 *
 * For every sequence b, head h and packed row p < n_packed[b]:
 *   out[b,h,p,:] = softmax over { context keys c < ctx_len[b] } U { packed keys q with
 *   tree_mask bit (p,q) set } of scale * <q[b,h,p,:], key>, applied to the values.
 * Keys outside that set do not take part (they are excluded, not biased).  Rows
 * p >= n_packed[b] of `out` are written as zero.  Cache entries at positions
 * >= ctx_len[b] and packed rows >= n_packed[b] are never read.
 *
 *   q, k_new, v_new, out : [B,H,N,D]      k_cache, v_cache : [B,H,Cmax,D]
 *   element type by `dt`: RD_F32 (float), RD_BF16 (bfloat16) or RD_F16 (IEEE half; the paper's
 *   App. A.2 runs its drafting in float16); scores and accumulation are fp32 in all three; all
 *   tensor pointers 16-byte aligned.
 *   ctx_len, n_packed : int32 [B];  tree_mask_bits : uint64 [B,N,ceil(N/64)] (rd_dedup's).
 *   Cmax >= 0 (k_cache/v_cache may be NULL when Cmax == 0).
 *
 * workspace: device scratch of at least rd_tree_attn_workspace(...) bytes, 256-byte
 * aligned.  It holds per-split partial results and completion counters.  The workspace
 * must be all zero before the first call that uses it (hipMemsetAsync it once); every
 * call leaves the counters zero again, so successive calls WITH THE SAME SHAPE ARGUMENTS
 * on one stream can reuse it without clearing.  Its layout depends on the shape: clear it
 * again before using it with other shape arguments.  Concurrent calls need separate
 * workspaces.  If a call fails or is aborted, clear the workspace before reusing it.
 */
size_t rd_tree_attn_workspace(int B, int H, int N, int D, int Cmax, rd_dtype dt);

int rd_tree_attn(const void *q, const void *k_cache, const void *v_cache,
                 const int32_t *ctx_len, const void *k_new, const void *v_new,
                 const int32_t *n_packed, const uint64_t *tree_mask_bits,
                 int B, int H, int N, int D, int Cmax, rd_dtype dt, float scale,
                 void *out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * rd_tree_attn_bounded — rd_tree_attn for a cache whose capacity is far above the live contexts (a
 * serving system allocates Cmax for the longest sequence it admits; Sec. 4.1's batches hold much shorter
 * ones).  rd_tree_attn chooses how many workgroups share a head from Cmax, the only length the host
 * knows; here the caller, who tracks sequence lengths, supplies ctx_bound, an upper bound of
 * ctx_len[b] over the batch for this call, and the plan is made for that.  The bound only steers the
 * plan: a sequence longer than ctx_bound is still computed in full, just with a plan that suits it
 * less; values above Cmax mean Cmax.  Results are those of rd_tree_attn.
 * workspace: at least rd_tree_attn_workspace(B, H, N, D, min(ctx_bound, Cmax), dt) bytes -- for a
 * workspace shared by calls with different bounds, the largest of these -- otherwise as for
 * rd_tree_attn (the zero-before-first-use contract does not depend on the bound: every call leaves the
 * counters zero and they sit at the same place for every bound).
 */
int rd_tree_attn_bounded(const void *q, const void *k_cache, const void *v_cache,
                         const int32_t *ctx_len, const void *k_new, const void *v_new,
                         const int32_t *n_packed, const uint64_t *tree_mask_bits,
                         int B, int H, int N, int D, int Cmax, int ctx_bound, rd_dtype dt, float scale,
                         void *out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * rd_tree_attn_rope — rd_tree_attn with the rotary position embedding of the packed candidates applied
 * inside the call instead of by a separate rd_rope launch (the paper's LLMs, Vicuna, Sec. 4, are
 * LLaMA-family models whose attention rotates queries and keys; a packed token sits at position
 * ctx_len + depth, rd_dedup's position_ids).  q and k_new arrive UNROTATED; the context keys in k_cache
 * are rotated already, as such a model's cache holds them.  The result equals rd_rope on (q, k_new)
 * followed by rd_tree_attn, bit for bit: the rotation uses rd_rope's arithmetic and rounds to the
 * storage type before the scores.
 *
 *   position_ids : int32 [B,N];  cos_tab, sin_tab : float [max_pos, D/2];  positions are clamped to
 *   [0, max_pos-1] (all as for rd_rope).
 *   k_new_rot : [B,H,N,D] of the element type, or NULL: receives the rotated rows p < n_packed[b] of
 *   k_new (what rd_commit has to append to the cache); rows beyond are left untouched.  Must not be
 *   k_new or q themselves (workgroups still read the unrotated rows while others write).
 *   dt = RD_BF16 or RD_F16.  Everything else, the workspace included (rd_tree_attn_workspace), as for
 *   rd_tree_attn.
 */
int rd_tree_attn_rope(const void *q, const void *k_cache, const void *v_cache,
                      const int32_t *ctx_len, const void *k_new, const void *v_new,
                      const int32_t *n_packed, const uint64_t *tree_mask_bits,
                      const int32_t *position_ids, const float *cos_tab, const float *sin_tab, int max_pos,
                      int B, int H, int N, int D, int Cmax, rd_dtype dt, float scale,
                      void *out, void *k_new_rot, void *workspace, size_t workspace_bytes, void *stream);

/*
 * rd_tree_attn_paged — rd_tree_attn with the context keys and values held in fixed-size pages, the
 * cache layout of serving systems built on paged attention (the production inference framework
 * the paper reports on in Sec. 4.1 and its acknowledgements is one).  Same computation and outputs as rd_tree_attn.
 *
 *   k_pages, v_pages : [n_pages, H, page_size, D], bf16 or fp16 (dt = RD_BF16 / RD_F16 only)
 *   block_table      : int32 [B, max_pages]; entry j of row b is the page that holds context keys
 *                      j*page_size .. (j+1)*page_size-1 of sequence b.  Only entries below
 *                      ceil(ctx_len[b] / page_size) are read; values are clamped to [0, n_pages-1].
 *   page_size        : keys per page, a multiple of 32;  ctx_len[b] <= page_size * max_pages.
 *   q, k_new, v_new, out, ctx_len, n_packed, tree_mask_bits, scale, workspace: as for rd_tree_attn
 *   (workspace size from rd_tree_attn_paged_workspace; same zero-before-first-use contract).
 */
size_t rd_tree_attn_paged_workspace(int B, int H, int N, int D, int page_size, int max_pages, rd_dtype dt);

int rd_tree_attn_paged(const void *q, const void *k_pages, const void *v_pages,
                       const int32_t *block_table, int page_size, int max_pages, int n_pages,
                       const int32_t *ctx_len, const void *k_new, const void *v_new,
                       const int32_t *n_packed, const uint64_t *tree_mask_bits,
                       int B, int H, int N, int D, rd_dtype dt, float scale,
                       void *out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * rd_accept — greedy verification (Sec. 3.4, Fig. 2; temperature 0).
 *
 *   argmax_out[b][p] = arg max_v logits[b][p][v] for p < n_packed[b] (smallest v among
 *                      equal maxima), -1 for p >= n_packed[b].  Row p is the LLM's
 *                      output at packed token p, i.e. its prediction of the token
 *                      that follows p on p's path.
 *   Candidate w's token j is accepted iff tokens 0..j-1 were and
 *       j == 0: root_token == NULL (the first token is the LLM's guaranteed one), or
 *               beams[b][w][0] == root_token[b];
 *       j >= 1: argmax_out[b][unpack_index[b][w][j-1]] == beams[b][w][j].
 *   n_accept[b][w]  length of candidate w's accepted prefix
 *   best_len[b]     max over w;  best_beam[b] = smallest w reaching it
 *   accepted_idx[b][t] = unpack_index[b][best_beam][t] for t < best_len (pad -1)
 *   next_token[b]   argmax_out at the last accepted slot; root_token[b] if best_len == 0
 *
 * logits: float [B,N,V], free of NaN (-inf allowed).  beams, unpack_index: int32
 * [B,W,L]; n_packed: int32 [B]; root_token: int32 [B] or NULL.  Outputs int32:
 * argmax_out [B,N], n_accept [B,W], best_beam/best_len/next_token [B],
 * accepted_idx [B,L].  logits must be 16-byte aligned.
 *
 * workspace: as for rd_tree_attn (at least rd_accept_workspace(...) bytes, 256-byte
 * aligned, all zero before first use, counters left zero by every call, tied to the
 * shape arguments).
 */
size_t rd_accept_workspace(int B, int W, int L, int V);

int rd_accept(const float *logits, const int32_t *beams, const int32_t *unpack_index,
              const int32_t *n_packed, const int32_t *root_token,
              int B, int W, int L, int V,
              int32_t *argmax_out, int32_t *n_accept, int32_t *best_beam,
              int32_t *best_len, int32_t *next_token, int32_t *accepted_idx,
              void *workspace, size_t workspace_bytes, void *stream);

/*
 * rd_accept_static — rd_accept for callers that cannot allocate device memory or pass a workspace:
 * code running under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, outputs and kernel as rd_accept, minus the workspace: the counters and row keys live in
 * a device array inside the library, RD_ACCEPT_STATIC_BYTES (1 MiB) per GPU, held by every GPU the
 * library runs on until the process ends.  The call allocates nothing and frees nothing (on a GPU's
 * first call it looks up the array's address once; a caller that captures graphs makes one call on
 * that GPU before the capture begins) and enqueues two kernels on `stream`: one that
 * clears the part of the array the call uses, then rd_accept's.
 *
 * Sizes with rd_accept_workspace(B, W, L, V) > RD_ACCEPT_STATIC_BYTES (about B*W*L > 87000 packed rows)
 * are rejected with RD_ERR_SCRATCH_LIMIT before anything is launched; the other argument errors are
 * rd_accept's.  All calls on one GPU share that GPU's array: calls that may overlap on one GPU (two
 * streams, two threads) race and must be serialised by the caller, or use rd_accept with separate
 * workspaces.
 */
#define RD_ACCEPT_STATIC_BYTES (1 << 20)

int rd_accept_static(const float *logits, const int32_t *beams, const int32_t *unpack_index,
                     const int32_t *n_packed, const int32_t *root_token,
                     int B, int W, int L, int V,
                     int32_t *argmax_out, int32_t *n_accept, int32_t *best_beam,
                     int32_t *best_len, int32_t *next_token, int32_t *accepted_idx, void *stream);

/*
 * rd_accept_sample — acceptance by rejection sampling, the selection mode Sec. 3.4 names for
 * sampling at a temperature.  The paper gives no procedure; this is speculative sampling as
 * published (Leviathan et al.; Chen et al., 2023), applied to every candidate on the packed tree.
 *
 *   p_s = softmax(logits[b][s] / temperature), the LLM's distribution after packed token s;
 *   q_s = softmax(draft_logits[b][s]), the draft model's distribution at the same place.
 *   Candidate w's token j >= 1 (x = beams[b][w][j], under slot s = unpack_index[b][w][j-1], stored in
 *   slot c = unpack_index[b][w][j]) is accepted, given tokens 0..j-1 were, iff
 *       u_accept[b][c] < min(1, p_s(x) / q_s(x))
 *   (one uniform number per packed slot: candidates that share a prefix share its decisions; a
 *   token outside [0, V) is rejected).  Token 0 as in rd_accept (root_token).
 *   n_accept, best_beam (longest accepted prefix, smallest index among equals), best_len,
 *   accepted_idx as in rd_accept.
 *   next_token[b]: drawn by inverting the cumulative distribution with u_next[b] — the smallest v
 *   with sum_{v' <= v} weight(v') > u_next[b] * sum weight and weight(v) > 0 — where weight = p_s
 *   at the candidate's last slot when it was accepted whole, else the residual max(0, p_s - q_s) at
 *   the slot s under which its first rejected token hangs (p_s if the residual vanishes);
 *   root_token[b] if best_len == 0.
 *
 * Arithmetic is fp32: a decision whose u lies within ~1e-5 of its threshold, or of a step of the
 * cumulative distribution, may differ from an exact evaluation.
 *
 * logits, draft_logits : float [B,N,V], 16-byte aligned, free of NaN, at least one finite entry per
 * row that is read.  Rows p >= n_packed[b] are not read; draft_logits rows of slots at the last
 * position (depth L-1) are not read either (the draft model has no distribution there).
 * draft_step_row : NULL, or int32 [B][W][L-1] = rd_draft's step_row: then draft_logits is rd_draft's
 * step_logits, float [L-1][draft_rows_per_step][V] (draft_rows_per_step = the B*W of that call), and the
 * draft distribution after candidate w's token j is row draft_step_row[b][w][j] of matrix j; no copy
 * into the packed layout is needed.  Row numbers are clamped to the matrix.
 * u_accept : float [B,N] in [0,1);  u_next : float [B] in [0,1);  temperature > 0.
 * beams, unpack_index, n_packed, root_token and the int32 outputs as for rd_accept (no argmax_out).
 * workspace: as for rd_accept (at least rd_accept_sample_workspace(...) bytes, 256-byte aligned, all
 * zero before first use, counters left zero by every call, not shared by concurrent calls).
 * V <= 1048576.  Two launches on `stream`.
 */
size_t rd_accept_sample_workspace(int B, int W, int L, int V);

int rd_accept_sample(const float *logits, const float *draft_logits, const int32_t *draft_step_row,
                     int draft_rows_per_step, const int32_t *beams, const int32_t *unpack_index, const int32_t *n_packed, const int32_t *root_token,
                     const float *u_accept, const float *u_next, float temperature,
                     int B, int W, int L, int V,
                     int32_t *n_accept, int32_t *best_beam, int32_t *best_len, int32_t *next_token,
                     int32_t *accepted_idx, void *workspace, size_t workspace_bytes, void *stream);

/*
 * rd_commit — the accepted tokens join the sequence generated so far (last step of the decoding
 * loop of Sec. 3.4; the LLM's hidden state at the last accepted token and next_token start the
 * next draft).  Runs after rd_accept, on its outputs.
 *
 * For every sequence b, with bl = best_len[b] clamped to [0, L], c = ctx_len[b] clamped to
 * [0, Cmax] and n = min(bl, Cmax - c) (what still fits in the cache):
 *   k_cache[b,h,c+t,:] = k_new[b,h,accepted_idx[b][t],:]   for t < n and every head h
 *   v_cache likewise;  rows are copied bit for bit
 *   ctx_len_out[b] = c + n;   n_committed[b] = n (a caller sees n < best_len[b] when the
 *   cache is full)
 *   hidden_last[b,:] = hidden[b, accepted_idx[b][bl-1], :]  if bl > 0, else left unchanged
 * Slots in accepted_idx are clamped to [0, N-1].  Nothing else in the caches is touched.
 *
 *   k_new, v_new : [B,H,N,D];  k_cache, v_cache : [B,H,Cmax,D] (updated in place), element
 *   type by `dt` as for rd_tree_attn, all 16-byte aligned.
 *   accepted_idx : int32 [B,L];  best_len, ctx_len : int32 [B];  ctx_len_out : int32 [B],
 *   must not overlap ctx_len (workgroups read ctx_len while another writes the new value:
 *   keep two arrays and alternate).  n_committed : int32 [B] or NULL.
 *   hidden : [B,N,Dh] and hidden_last : [B,Dh] of the same element type, 16-byte aligned,
 *   Dh * element size a multiple of 16; both NULL (and Dh = 0) to skip.
 * No workspace.  D in {64, 128} as for rd_tree_attn; Cmax >= 1.
 */
int rd_commit(const void *k_new, const void *v_new, const int32_t *accepted_idx,
              const int32_t *best_len, const int32_t *ctx_len,
              int B, int H, int N, int D, int Cmax, int L, rd_dtype dt,
              void *k_cache, void *v_cache, int32_t *ctx_len_out, int32_t *n_committed,
              const void *hidden, int Dh, void *hidden_last, void *stream);

/*
 * rd_rope — rotary position embedding of the packed candidates, at the positions rd_dedup produced.
 * The paper leaves positions to the LLM; its LLMs (Vicuna, Sec. 4) are LLaMA-family models whose
 * attention rotates queries and keys, and a packed token sits at position ctx_len + depth
 * (rd_dedup's position_ids).  Run it on q and k_new before rd_tree_attn (and rd_commit then stores
 * rotated keys, as such a model's cache holds them).
 *
 * For b, h, packed row p < n_packed[b], pos = position_ids[b][p] clamped to [0, max_pos-1], i < D/2:
 *     y[i]       = x[i] * cos_tab[pos][i] - x[i + D/2] * sin_tab[pos][i]
 *     y[i + D/2] = x[i + D/2] * cos_tab[pos][i] + x[i] * sin_tab[pos][i]
 * ("rotate half" pairing), computed in fp32 with every product rounded before the sum, rounded once
 * to the storage type, in place.  Rows p >= n_packed[b] are left untouched.
 *
 *   q, k_new : [B,H,N,D], element type by `dt` (any of the three), 32-byte aligned; either may be
 *   NULL (skipped).  position_ids : int32 [B,N];  n_packed : int32 [B].
 *   cos_tab, sin_tab : float [max_pos, D/2], cos / sin of pos * theta_i for whatever base and
 *   scaling the model uses (the library does no trigonometry).
 */
int rd_rope(void *q, void *k_new, const int32_t *position_ids, const int32_t *n_packed,
            const float *cos_tab, const float *sin_tab, int max_pos,
            int B, int H, int N, int D, rd_dtype dt, void *stream);

/*
 * rd_commit_paged — rd_commit for the paged cache of rd_tree_attn_paged: position p of sequence b is
 * row p % page_size of page block_table[b][p / page_size] (pages [n_pages, H, page_size, D]); the
 * capacity per sequence is page_size * max_pages.  The caller must have entered pages into the block
 * table for every position that can be written (ctx_len[b] .. ctx_len[b] + L - 1); entries are
 * clamped to [0, n_pages-1].  Everything else as for rd_commit (any page_size > 0; fp32 pages are
 * accepted here although rd_tree_attn_paged reads 16-bit pages only).
 */
int rd_commit_paged(const void *k_new, const void *v_new, const int32_t *accepted_idx,
                    const int32_t *best_len, const int32_t *ctx_len,
                    int B, int H, int N, int D, int L, rd_dtype dt,
                    void *k_pages, void *v_pages, const int32_t *block_table,
                    int page_size, int max_pages, int n_pages,
                    int32_t *ctx_len_out, int32_t *n_committed,
                    const void *hidden, int Dh, void *hidden_last, void *stream);

/*
 * rd_draft — the draft model and its beam search (Sec. 3.1, 3.2): produces the W candidates of
 * length L that rd_dedup takes, from the LLM's last hidden state and latest token.
 *
 *   s_1 = e(last_token);  at drafted position t = 1 .. L-1, for every live candidate:
 *     g = [s_t, h];  x = g;  x <- x + f(A_k x + c_k) for k < n_mlp;  log p = log_softmax(O x)
 *   the best W (candidate, token) pairs by cumulative log probability survive (ties: smaller
 *   candidate, then smaller token; at t = 1 there is one state, so they are its W most probable
 *   tokens), and s_{t+1} = f(U s_t[parent] + W e(token) + b).  f = SiLU (the paper names none).
 *   beams[b][w] = [last_token[b], token_1, ..., token_{L-1}], best candidate first;
 *   beam_logp[b][w] = its cumulative log probability (0 when L == 1).
 *
 * Precision: weights, embeddings and h are bf16 (or fp16, params.dtype; the paper's MLX runs draft in
 * float16, App. A.2); every linear layer reads its input rounded to that type and accumulates in fp32; biases, activation, skip connection, log-softmax, scores fp32.
 * Two candidates whose scores differ by less than that arithmetic resolves may swap places
 * against an exact evaluation.
 *
 * rd_draft_params (a HOST struct of DEVICE pointers, all weights row-major [out][in], 16-byte
 * aligned): emb [V,Dm]; rnn_u, rnn_w [Dm,Dm]; rnn_b float [Dm]; mlp_w [n_mlp,2Dm,2Dm]; mlp_b float
 * [n_mlp,2Dm]; head_w [V,2Dm]; the matrices and emb in the 16-bit type `dtype`.
 * h : that type, [B,Dm];  last_token : int32 [B] (clamped to [0, V-1]);  beams : int32 [B,W,L];
 * beam_logp : float [B,W].
 * step_logits, step_row : both NULL, or the record of the search that rd_accept_sample takes:
 *   step_logits float [L-1][B*W][V], 16-byte aligned: the output layer's values (softmax of a row = the
 *   draft distribution) of every live candidate at every drafted position, row b*W + w of matrix t-1
 *   = live candidate w of sequence b at position t (at position 1 only w = 0 is live; other rows
 *   of that matrix are not written);
 *   step_row int32 [B][W][L-1]: the row of matrix t-1 that produced token t of final candidate w.  workspace: rd_draft_workspace(...) bytes, 256-byte aligned, no
 * initial contents required, not shared by concurrent calls.
 * Limits: Dm a multiple of 64; W <= 128, W <= V; B*W <= 512; V <= 262144; L <= 384.
 * The call enqueues at most 4 + n_mlp launches per drafted position (5 + n_mlp after the first; one
 * fewer for W <= 8 and V <= 32768) while B*W <= 128; every further 128 rows add one launch per linear layer.
 */
typedef struct {
    const void *emb, *rnn_u, *rnn_w;
    const float *rnn_b;
    const void *mlp_w;
    const float *mlp_b;
    const void *head_w;
    int n_mlp, Dm, V;
    rd_dtype dtype;          /* RD_BF16 or RD_F16: type of emb, rnn_u, rnn_w, mlp_w, head_w and of h */
    int tiled;               /* 0: the matrices are row-major; 1: rnn_u, rnn_w, every mlp_w[k] and head_w are in
                                the layout rd_draft_pack_weights writes (emb stays row-major) */
} rd_draft_params;

/*
 * rd_draft_pack_weights — one-time layout change of a weight matrix for rd_draft (at model load).
 * src: [N][K] row-major, 16-bit elements (bf16 or fp16, copied bit for bit), K a multiple of 32.
 * dst: rd_draft_packed_elems(N, K) elements = ceil(N/16)*16 * K: tiles of 16 rows x 32 columns, tile
 * (n/16, k/32) stored as the 1 KB a wave loads for one matrix-core operand (element (n, k) at
 * ((n/16 * K/32 + k/32) * 64 + ((k%32)/8) * 16 + n%16) * 8 + k%8), rows past N zero.  With this layout
 * every wave load of the linear layers reads 1 KB of consecutive memory; results are bit-identical to
 * the row-major layout.  Each of the n_mlp matrices of mlp_w is packed on its own, back to back.
 * Both pointers 16-byte aligned, src and dst must not overlap.
 */
size_t rd_draft_packed_elems(int N, int K);
int rd_draft_pack_weights(const void *src, int N, int K, void *dst, void *stream);

size_t rd_draft_workspace(int B, int W, int L, int Dm, int V);

int rd_draft(const rd_draft_params *p, const void *h, const int32_t *last_token,
             int B, int W, int L, int32_t *beams, float *beam_logp,
             float *step_logits, int32_t *step_row,
             void *workspace, size_t workspace_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* RD_H */
