/*
 * CPU oracle for the ReDrafter verification step.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, definition-level implementation of what the verification step
 * computes (dynamic tree attention, Sec. 3.3 and App. A.1; verification, greedy and
 * rejection-sampling acceptance and the commit of the accepted tokens, Sec. 3.4) and of the
 * draft model with its beam search (Sec. 3.1, 3.2).  It exists so that
 * the HIP path can be checked against something that is easy to compare with the
 * paper by eye.  It shares no code
 * with the HIP path and must never be called from it; only tests, the smoke
 * check and the benchmark's CPU-baseline leg use it.
 *
 * Everything here is per sequence; a batch is B independent sequences
 * (App. A.1: a batch dimension is simply prepended).
 *
 * Floating point: inputs are upcast exactly to double, all arithmetic is double,
 * the result is rounded once (round-to-nearest-even) to the storage type.
 *
 * Every function in this file is pinned by tests that do not use this file's
 * own arithmetic (the worked example of App. A.1, a literal prefix trie, closed
 * forms, per-beam causal attention in numpy, library argmax, a toy greedy LM; for the
 * draft model: a numpy/scipy forward pass, greedy decoding, exhaustive search; for the
 * commit: numpy index arithmetic, attention over the committed cache, and a many-step
 * speculative loop that must reproduce plain greedy decoding of a toy attention LM; for
 * the rejection-sampling acceptance: the published guarantee that the emitted token follows
 * the LLM's distribution with acceptance rate sum min(p, q), the zero-temperature limit,
 * identical models, library softmax / cumsum / searchsorted, a walk over a literal trie).
 *
 * OpenMP (if enabled at compile time) parallelises only over independent
 * (sequence, head) pairs or logit rows; the arithmetic per output is unchanged.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_F32 0
#define ORC_BF16 1
#define ORC_F16 2

int orc_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------- */
/* dedup_prefix (App. A.1): prefix_tree[i][j] is the smallest candidate index k
 * whose first j+1 tokens equal candidate i's first j+1 tokens.               */
/* ------------------------------------------------------------------------- */
void orc_dedup_prefix(const int32_t *beam, int W, int L, int32_t *prefix_tree)
{
    for (int i = 0; i < W; ++i) {
        for (int j = 0; j < L; ++j) {
            int found = i;
            for (int k = 0; k <= i; ++k) {
                int same = 1;
                for (int t = 0; t <= j; ++t)
                    if (beam[k * L + t] != beam[i * L + t]) same = 0;
                if (same) { found = k; break; }
            }
            prefix_tree[i * L + j] = found;
        }
    }
}

/* ------------------------------------------------------------------------- */
/* pack_beam (Sec. 3.3, App. A.1): a token can be condensed away when
 * prefix_tree[i][j] < i, so the kept ones are those with prefix_tree[i][j] == i.
 * Kept tokens are numbered in row-major (candidate, position) order.
 * Outputs (N = W*L entries each, padded with -1 beyond the packed count P):
 *   packed_tokens[p], src_beam[p], depth[p];  unpack_index[i][j] = packed slot
 *   that holds candidate i's j-th token.  Returns P.                          */
/* ------------------------------------------------------------------------- */
int orc_pack_beam(const int32_t *beam, const int32_t *prefix_tree, int W, int L,
                  int32_t *packed_tokens, int32_t *src_beam, int32_t *depth,
                  int32_t *unpack_index)
{
    const int N = W * L;
    int32_t *slot = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
    int P = 0;
    for (int i = 0; i < W; ++i)
        for (int j = 0; j < L; ++j) {
            if (prefix_tree[i * L + j] == i) {
                slot[i * L + j] = P;
                packed_tokens[P] = beam[i * L + j];
                src_beam[P] = i;
                depth[P] = j;
                ++P;
            } else {
                slot[i * L + j] = -1;
            }
        }
    for (int p = P; p < N; ++p) {
        packed_tokens[p] = -1;
        src_beam[p] = -1;
        depth[p] = -1;
    }
    for (int i = 0; i < W; ++i)
        for (int j = 0; j < L; ++j)
            unpack_index[i * L + j] = slot[prefix_tree[i * L + j] * L + j];
    free(slot);
    return P;
}

/* ------------------------------------------------------------------------- */
/* Tree structure of the packed beam (Sec. 3.3, Fig. 3): a packed token depends
 * on the packed tokens that hold the earlier positions of its own candidate,
 * and on itself.  ctx_len < 0 means "no context": position ids are depths.    */
/* ------------------------------------------------------------------------- */
void orc_tree_structure(const int32_t *unpack_index, const int32_t *src_beam,
                        const int32_t *depth, int P, int W, int L, int ctx_len,
                        int32_t *parent, int32_t *position_ids,
                        uint8_t *tree_mask /* [N,N] */,
                        uint64_t *tree_mask_bits /* [N, ceil(N/64)] */)
{
    const int N = W * L;
    const int words = (N + 63) / 64;
    memset(tree_mask, 0, (size_t)N * (size_t)N);
    memset(tree_mask_bits, 0, sizeof(uint64_t) * (size_t)N * (size_t)words);
    for (int p = 0; p < N; ++p) {
        if (p >= P) { parent[p] = -1; position_ids[p] = -1; continue; }
        const int i = src_beam[p];
        const int j = depth[p];
        parent[p] = (j == 0) ? -1 : unpack_index[i * L + (j - 1)];
        position_ids[p] = (ctx_len < 0 ? 0 : ctx_len) + j;
        for (int t = 0; t <= j; ++t) {
            const int q = unpack_index[i * L + t];
            tree_mask[(size_t)p * N + q] = 1;
            tree_mask_bits[(size_t)p * words + (q >> 6)] |= (uint64_t)1 << (q & 63);
        }
    }
}

/* Batched front end for the three integer steps above. */
void orc_dedup(const int32_t *beams /*[B,W,L]*/, const int32_t *ctx_len /*[B] or NULL*/,
               int B, int W, int L,
               int32_t *prefix_tree, int32_t *packed_tokens, int32_t *n_packed,
               int32_t *unpack_index, int32_t *parent, int32_t *position_ids,
               uint8_t *tree_mask, uint64_t *tree_mask_bits)
{
    const int N = W * L;
    const int words = (N + 63) / 64;
    int32_t *src_beam = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
    int32_t *depth = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
    for (int b = 0; b < B; ++b) {
        const int32_t *beam = beams + (size_t)b * N;
        int32_t *pt = prefix_tree + (size_t)b * N;
        int32_t *ui = unpack_index + (size_t)b * N;
        orc_dedup_prefix(beam, W, L, pt);
        const int P = orc_pack_beam(beam, pt, W, L, packed_tokens + (size_t)b * N,
                                    src_beam, depth, ui);
        n_packed[b] = P;
        orc_tree_structure(ui, src_beam, depth, P, W, L, ctx_len ? ctx_len[b] : -1,
                           parent + (size_t)b * N, position_ids + (size_t)b * N,
                           tree_mask + (size_t)b * N * N,
                           tree_mask_bits + (size_t)b * N * words);
    }
    free(src_beam);
    free(depth);
}

/* ------------------------------------------------------------------------- */
/* storage formats                                                             */
/* ------------------------------------------------------------------------- */
static double load_elem(const void *base, size_t idx, int dtype)
{
    if (dtype == ORC_BF16) {
        uint32_t u = (uint32_t)((const uint16_t *)base)[idx] << 16;
        float f;
        memcpy(&f, &u, 4);
        return (double)f;
    }
    if (dtype == ORC_F16) {
        /* IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits */
        const uint16_t h = ((const uint16_t *)base)[idx];
        const int sign = h >> 15, e = (h >> 10) & 31, frac = h & 1023;
        double v;
        if (e == 31) v = frac ? NAN : INFINITY;
        else if (e == 0) v = ldexp((double)frac, -24);              /* subnormal or zero */
        else v = ldexp(1.0 + (double)frac / 1024.0, e - 15);
        return sign ? -v : v;
    }
    return (double)((const float *)base)[idx];
}

static uint16_t double_to_bf16(double x)
{
    /* one rounding, ties to even, from the double straight to 8 significand bits */
    if (isnan(x)) return 0x7FC0;
    float f;
    if (isinf(x) || x == 0.0) {
        f = (float)x;
    } else {
        int e;
        (void)frexp(fabs(x), &e);          /* |x| = m * 2^e with m in [0.5, 1) */
        int qexp = e - 8;                  /* exponent of the last kept bit */
        if (qexp < -133) qexp = -133;      /* bf16 subnormal spacing */
        const double r = nearbyint(ldexp(x, -qexp));   /* default mode: ties to even */
        f = (float)ldexp(r, qexp);         /* exact, or +-inf on overflow */
    }
    uint32_t u;
    memcpy(&u, &f, 4);
    return (uint16_t)(u >> 16);
}

static uint16_t double_to_f16(double x)
{
    /* one rounding, ties to even, from the double straight to 11 significand bits */
    const uint16_t sign = signbit(x) ? 0x8000 : 0;
    if (isnan(x)) return 0x7E00;
    const double ax = fabs(x);
    if (isinf(ax)) return sign | 0x7C00;
    if (ax == 0.0) return sign;
    int e;
    (void)frexp(ax, &e);                    /* ax = m * 2^e with m in [0.5, 1) */
    int qexp = e - 11;                      /* exponent of the last kept bit */
    if (qexp < -24) qexp = -24;             /* subnormal spacing */
    const double r = nearbyint(ldexp(ax, -qexp));      /* integer in [0, 2048] */
    const double v = ldexp(r, qexp);
    if (v >= 65520.0) return sign | 0x7C00; /* rounds past the largest finite half (65504) */
    if (v == 0.0) return sign;
    int e2;
    const double m2 = frexp(v, &e2);        /* v = m2 * 2^e2, exact */
    if (e2 - 1 < -14)                       /* subnormal: fraction field = v / 2^-24 */
        return sign | (uint16_t)ldexp(v, 24);
    const uint16_t frac = (uint16_t)(ldexp(m2, 11) - 1024.0);       /* m2*2 in [1,2): 10 fraction bits */
    return sign | (uint16_t)((e2 - 1 + 15) << 10) | frac;
}

static void store_elem(void *base, size_t idx, int dtype, double x)
{
    if (dtype == ORC_F16) { ((uint16_t *)base)[idx] = double_to_f16(x); return; }
    if (dtype == ORC_BF16) ((uint16_t *)base)[idx] = double_to_bf16(x);
    else ((float *)base)[idx] = (float)x;
}

/* ------------------------------------------------------------------------- */
/* Tree-masked attention of one packed token (Sec. 3.3/3.4): softmax over all
 * context keys c < ctx_len and over the packed keys its mask row allows, of
 * scale * <q_p, k>, applied to the values.  Masked keys are absent from the
 * softmax.  Result in out_row[0..D).                                          */
/* ------------------------------------------------------------------------- */
static void attn_row(const void *q, const void *k_cache, const void *v_cache,
                     const void *k_new, const void *v_new, const uint8_t *mask_row,
                     int ctx, int P, int N, int D, int Cmax, int dtype, double scale,
                     size_t bh, int p, double *s /* [Cmax+N] */, double *out_row)
{
    const size_t qoff = (bh * (size_t)N + (size_t)p) * (size_t)D;
    const size_t cbase = bh * (size_t)Cmax * (size_t)D;
    const size_t nbase = bh * (size_t)N * (size_t)D;
    int n = 0;
    double m = -INFINITY;
    for (int c = 0; c < ctx; ++c) {
        double dot = 0.0;
        for (int d = 0; d < D; ++d)
            dot += load_elem(q, qoff + d, dtype) * load_elem(k_cache, cbase + (size_t)c * D + d, dtype);
        s[n] = scale * dot;
        if (s[n] > m) m = s[n];
        ++n;
    }
    for (int t = 0; t < P; ++t) {
        if (!mask_row[t]) continue;
        double dot = 0.0;
        for (int d = 0; d < D; ++d)
            dot += load_elem(q, qoff + d, dtype) * load_elem(k_new, nbase + (size_t)t * D + d, dtype);
        s[n] = scale * dot;
        if (s[n] > m) m = s[n];
        ++n;
    }
    double denom = 0.0;
    for (int d = 0; d < D; ++d) out_row[d] = 0.0;
    n = 0;
    for (int c = 0; c < ctx; ++c) {
        const double w = exp(s[n++] - m);
        denom += w;
        for (int d = 0; d < D; ++d)
            out_row[d] += w * load_elem(v_cache, cbase + (size_t)c * D + d, dtype);
    }
    for (int t = 0; t < P; ++t) {
        if (!mask_row[t]) continue;
        const double w = exp(s[n++] - m);
        denom += w;
        for (int d = 0; d < D; ++d)
            out_row[d] += w * load_elem(v_new, nbase + (size_t)t * D + d, dtype);
    }
    for (int d = 0; d < D; ++d) out_row[d] /= denom;
}

static int clampi(int x, int lo, int hi) { return x < lo ? lo : (x > hi ? hi : x); }

/* Whole tensor: out [B,H,N,D] in the storage dtype; rows p >= n_packed[b] are zero. */
void orc_tree_attn(const void *q, const void *k_cache, const void *v_cache,
                   const int32_t *ctx_len, const void *k_new, const void *v_new,
                   const int32_t *n_packed, const uint8_t *tree_mask /*[B,N,N]*/,
                   int B, int H, int N, int D, int Cmax, int dtype, float scale, void *out)
{
    const int BH = B * H;
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)(Cmax + N));
        double *row = (double *)malloc(sizeof(double) * (size_t)D);
#pragma omp for schedule(dynamic, 1)
        for (int bh = 0; bh < BH; ++bh) {
            const int b = bh / H;
            const int ctx = clampi(ctx_len[b], 0, Cmax);
            const int P = clampi(n_packed[b], 0, N);
            for (int p = 0; p < N; ++p) {
                const size_t ooff = ((size_t)bh * N + p) * (size_t)D;
                if (p >= P) {
                    for (int d = 0; d < D; ++d) store_elem(out, ooff + d, dtype, 0.0);
                    continue;
                }
                attn_row(q, k_cache, v_cache, k_new, v_new,
                         tree_mask + ((size_t)b * N + p) * N, ctx, P, N, D, Cmax, dtype,
                         (double)scale, (size_t)bh, p, s, row);
                for (int d = 0; d < D; ++d) store_elem(out, ooff + d, dtype, row[d]);
            }
        }
        free(s);
        free(row);
    }
}

/* Selected rows only: rows[r] = (b, h, p) with p < n_packed[b]; out_f64 [n_rows, D]
 * holds the unrounded double results (for spot checks on tensors too large to do whole). */
void orc_tree_attn_rows(const void *q, const void *k_cache, const void *v_cache,
                        const int32_t *ctx_len, const void *k_new, const void *v_new,
                        const int32_t *n_packed, const uint8_t *tree_mask,
                        int B, int H, int N, int D, int Cmax, int dtype, float scale,
                        const int32_t *rows, int n_rows, double *out_f64)
{
    (void)B;
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)(Cmax + N));
#pragma omp for schedule(dynamic, 1)
        for (int r = 0; r < n_rows; ++r) {
            const int b = rows[3 * r], h = rows[3 * r + 1], p = rows[3 * r + 2];
            const int ctx = clampi(ctx_len[b], 0, Cmax);
            const int P = clampi(n_packed[b], 0, N);
            attn_row(q, k_cache, v_cache, k_new, v_new, tree_mask + ((size_t)b * N + p) * N,
                     ctx, P, N, D, Cmax, dtype, (double)scale, (size_t)b * H + h, p, s,
                     out_f64 + (size_t)r * D);
        }
        free(s);
    }
}

/* ------------------------------------------------------------------------- */
/* Greedy verification (Sec. 3.4, temperature 0): the LLM's prediction after a
 * packed token is the arg max of that token's logit row (smallest index among
 * equal maxima); rows beyond the packed count give -1.                        */
/* ------------------------------------------------------------------------- */
void orc_argmax(const float *logits /*[B,N,V]*/, const int32_t *n_packed, int B, int N, int V,
                int32_t *argmax_out /*[B,N]*/)
{
    const int rows = B * N;
#pragma omp parallel for schedule(static)
    for (int r = 0; r < rows; ++r) {
        const int b = r / N, p = r % N;
        if (p >= n_packed[b]) { argmax_out[r] = -1; continue; }
        const float *row = logits + (size_t)r * V;
        int best = 0;
        for (int v = 1; v < V; ++v)
            if (row[v] > row[best]) best = v;
        argmax_out[r] = best;
    }
}

/* Token-match acceptance (Sec. 3.4, Fig. 2): candidate w's token j is accepted when
 * all earlier tokens were and the LLM's prediction after token j-1 equals it.  Token 0
 * is checked against root_token[b] (the LLM's already known next token) or, when
 * root_token is NULL, taken as given.  The best candidate has the longest accepted
 * prefix (smallest index among equals); next_token is the LLM's prediction after the
 * last accepted token.                                                         */
void orc_accept(const int32_t *beams, const int32_t *unpack_index, const int32_t *argmax_in,
                const int32_t *root_token, int B, int W, int L,
                int32_t *n_accept /*[B,W]*/, int32_t *best_beam, int32_t *best_len,
                int32_t *next_token, int32_t *accepted_idx /*[B,L]*/)
{
    const int N = W * L;
    for (int b = 0; b < B; ++b) {
        const int32_t *beam = beams + (size_t)b * N;
        const int32_t *ui = unpack_index + (size_t)b * N;
        const int32_t *am = argmax_in + (size_t)b * N;
        int bw = 0, bl = -1;
        for (int w = 0; w < W; ++w) {
            int len = 0;
            for (int j = 0; j < L; ++j) {
                int ok;
                if (j == 0) ok = (root_token == NULL) || (beam[w * L] == root_token[b]);
                else ok = (am[ui[w * L + j - 1]] == beam[w * L + j]);
                if (!ok) break;
                ++len;
            }
            n_accept[b * W + w] = len;
            if (len > bl) { bl = len; bw = w; }
        }
        best_beam[b] = bw;
        best_len[b] = bl;
        for (int t = 0; t < L; ++t)
            accepted_idx[b * L + t] = (t < bl) ? ui[bw * L + t] : -1;
        next_token[b] = (bl > 0) ? am[ui[bw * L + bl - 1]] : root_token[b];
    }
}

/* ---------------------------------------------------------------------------------
 * Commit of the accepted tokens (Sec. 3.4: the accepted tokens are appended to the
 * previously generated ones, and the LLM's hidden state at the last accepted token
 * seeds the next draft call).  For the attention path this means that the key and
 * value rows of the accepted packed tokens join the context:
 *     n = min(best_len[b], Cmax - ctx_len[b])            (what still fits)
 *     cache[b,h,ctx_len[b]+t,:] = new[b,h,accepted_idx[b][t],:]   for t < n, every h
 *     ctx_len_out[b] = ctx_len[b] + n,   n_committed[b] = n
 *     hidden_last[b,:] = hidden[b, accepted_idx[b][best_len[b]-1], :]  if best_len[b] > 0
 * Rows are copied bit for bit (no arithmetic).  best_len is clamped to [0, L], ctx_len
 * to [0, Cmax] and slots to [0, N-1]: the interface defines the step for out-of-range data this way.
 * n_committed, hidden / hidden_last may be NULL.                                   */
void orc_commit(const void *k_new, const void *v_new, const int32_t *accepted_idx,
                const int32_t *best_len, const int32_t *ctx_len,
                int B, int H, int N, int D, int Cmax, int L, int dtype,
                void *k_cache, void *v_cache, int32_t *ctx_len_out, int32_t *n_committed,
                const void *hidden, int Dh, void *hidden_last)
{
    const size_t es = (dtype == ORC_F32) ? 4 : 2;
    const size_t row = (size_t)D * es;
    for (int b = 0; b < B; ++b) {
        int bl = best_len[b];
        if (bl < 0) bl = 0;
        if (bl > L) bl = L;
        int ctx = ctx_len[b];
        if (ctx < 0) ctx = 0;
        if (ctx > Cmax) ctx = Cmax;
        const int n = (bl < Cmax - ctx) ? bl : Cmax - ctx;
        for (int t = 0; t < n; ++t) {
            int slot = accepted_idx[(size_t)b * L + t];
            if (slot < 0) slot = 0;
            if (slot > N - 1) slot = N - 1;
            for (int h = 0; h < H; ++h) {
                const size_t src = (((size_t)b * H + h) * N + slot) * row;
                const size_t dst = (((size_t)b * H + h) * Cmax + (size_t)(ctx + t)) * row;
                memcpy((unsigned char *)k_cache + dst, (const unsigned char *)k_new + src, row);
                memcpy((unsigned char *)v_cache + dst, (const unsigned char *)v_new + src, row);
            }
        }
        ctx_len_out[b] = ctx + n;
        if (n_committed) n_committed[b] = n;
        if (hidden && hidden_last && bl > 0) {
            int slot = accepted_idx[(size_t)b * L + bl - 1];
            if (slot < 0) slot = 0;
            if (slot > N - 1) slot = N - 1;
            memcpy((unsigned char *)hidden_last + (size_t)b * Dh * es,
                   (const unsigned char *)hidden + ((size_t)b * N + slot) * Dh * es, (size_t)Dh * es);
        }
    }
}

/* ---------------------------------------------------------------------------------
 * Rotary position embedding of the packed candidates.  The paper does not spell out
 * positions; with Vicuna (LLaMA family) as the LLM of Sec. 4, queries and keys carry
 * rotary embeddings, and a packed token's position is ctx_len + depth (position_ids
 * of the tree structure).  Convention: the LLaMA "rotate half" pairing, element i is
 * paired with element i + D/2 and the pair is rotated by the angle pos * theta_i whose
 * cosine and sine the caller supplies in tables [max_pos][D/2]:
 *     y[i]       = x[i] * cos[pos][i] - x[i + D/2] * sin[pos][i]
 *     y[i + D/2] = x[i + D/2] * cos[pos][i] + x[i] * sin[pos][i]
 * applied in place to rows p < n_packed[b] of x [B,H,N,D]; the result is rounded once
 * to the storage type.  pos is clamped to [0, max_pos - 1].                           */
void orc_rope(void *x, const int32_t *position_ids /*[B,N]*/, const int32_t *n_packed,
              const float *cos_tab, const float *sin_tab, int max_pos,
              int B, int H, int N, int D, int dtype)
{
    const int half = D / 2;
    double *y = (double *)malloc(sizeof(double) * (size_t)D);
    for (int b = 0; b < B; ++b) {
        int P = n_packed[b];
        if (P < 0) P = 0;
        if (P > N) P = N;
        for (int h = 0; h < H; ++h)
            for (int p = 0; p < P; ++p) {
                int pos = position_ids[(size_t)b * N + p];
                if (pos < 0) pos = 0;
                if (pos > max_pos - 1) pos = max_pos - 1;
                const size_t row = (((size_t)b * H + h) * N + p) * (size_t)D;
                for (int i = 0; i < half; ++i) {
                    const double c = (double)cos_tab[(size_t)pos * half + i];
                    const double s = (double)sin_tab[(size_t)pos * half + i];
                    const double lo = load_elem(x, row + i, dtype), hi = load_elem(x, row + i + half, dtype);
                    y[i] = lo * c - hi * s;
                    y[i + half] = hi * c + lo * s;
                }
                for (int d = 0; d < D; ++d) store_elem(x, row + d, dtype, y[d]);
            }
    }
    free(y);
}

/* ---------------------------------------------------------------------------------
 * The draft model and its beam search (Sec. 3.1, 3.2).  Per sequence:
 *   s_1 = e(last token)                    the embedding of the LLM's latest token
 *   g_t = [s_t, h]                         h = the LLM's last hidden state (Sec. 3.1)
 *   x = g_t;  x <- x + f(A_k x + c_k)      n_mlp residual MLP layers (Sec. 3.1)
 *   z = O x;  log p = log_softmax(z)       softmax output layer over the vocabulary
 *   s_{t+1} = f(U s_t + W e(token_t) + b)  the RNN update with the token chosen at step t
 * The paper names no activation f; SiLU is this build's reading (it is what the public
 * ReDrafter release uses).  Beam search of width W (Sec. 3.2) over T = L - 1 drafted
 * tokens, position 0 of every candidate being the LLM's own token: at each step the
 * candidates (beam w, token v) are ranked by cumulative log probability (ties: smaller w,
 * then smaller v) and the best W survive; at the first step there is one state, so the W
 * candidates are its W most probable tokens.
 *
 * Numerics (the precision contract shared with the device code): weights, embeddings and h
 * are bf16 (or float16, the type of the paper's MLX runs, App. A.2); every linear layer reads its
 * input vector rounded to that type and accumulates
 * without further rounding; biases, activation, skip connection, log-softmax and scores
 * are computed on unrounded values.  Here that arithmetic is double.
 * Weights are row-major [out][in]: rnn_u, rnn_w [Dm][Dm]; mlp_w [n_mlp][2Dm][2Dm];
 * head_w [V][2Dm]; emb [V][Dm].  Biases float.                                       */
static double bf16_to_double(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}
static double silu(double x) { return x / (1.0 + exp(-x)); }
/* the 16-bit storage type of the draft model: bf16 or, as in the paper's MLX runs (App. A.2), float16 */
static double w16_to_double(uint16_t v, int dtype)
{
    return dtype == ORC_F16 ? load_elem(&v, 0, ORC_F16) : bf16_to_double(v);
}
static double round16(double x, int dtype)
{
    return dtype == ORC_F16 ? w16_to_double(double_to_f16(x), ORC_F16) : bf16_to_double(double_to_bf16(x));
}

/* y[n] = sum_k round16(x[k]) * W[n][k] (+ bias[n]) */
static void linear16(const uint16_t *Wt, const float *bias, int N, int K, const double *x, double *y, int dtype)
{
    double *xr = (double *)malloc(sizeof(double) * (size_t)K);
    for (int k = 0; k < K; ++k) xr[k] = round16(x[k], dtype);
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        const uint16_t *row = Wt + (size_t)n * K;
        double acc = 0.0;
        for (int k = 0; k < K; ++k) acc += xr[k] * w16_to_double(row[k], dtype);
        y[n] = acc + (bias ? (double)bias[n] : 0.0);
    }
    free(xr);
}

/* log-probabilities of the next token given RNN state s and hidden h; lp has V entries */
static void draft_logp(const uint16_t *mlp_w, const float *mlp_b, int n_mlp, const uint16_t *head_w,
                       const double *s, const double *h, int Dm, int V, double *lp, int dtype)
{
    const int G = 2 * Dm;
    double *x = (double *)malloc(sizeof(double) * (size_t)G);
    double *y = (double *)malloc(sizeof(double) * (size_t)G);
    for (int i = 0; i < Dm; ++i) { x[i] = s[i]; x[Dm + i] = h[i]; }
    for (int k = 0; k < n_mlp; ++k) {
        linear16(mlp_w + (size_t)k * G * G, mlp_b ? mlp_b + (size_t)k * G : NULL, G, G, x, y, dtype);
        for (int i = 0; i < G; ++i) x[i] += silu(y[i]);
    }
    linear16(head_w, NULL, V, G, x, lp, dtype);
    double m = -INFINITY, sum = 0.0;
    for (int v = 0; v < V; ++v) if (lp[v] > m) m = lp[v];
    for (int v = 0; v < V; ++v) sum += exp(lp[v] - m);
    const double lse = m + log(sum);
    for (int v = 0; v < V; ++v) lp[v] -= lse;
    free(x);
    free(y);
}

/* s_next = f(U s + W e(token) + b) */
static void draft_rnn(const uint16_t *emb, const uint16_t *rnn_u, const uint16_t *rnn_w, const float *rnn_b,
                      const double *s, int token, int Dm, double *s_next, int dtype)
{
    double *e = (double *)calloc((size_t)Dm, sizeof(double));
    double *a = (double *)malloc(sizeof(double) * (size_t)Dm);
    double *c = (double *)malloc(sizeof(double) * (size_t)Dm);
    for (int i = 0; i < Dm; ++i) e[i] = w16_to_double(emb[(size_t)token * Dm + i], dtype);
    linear16(rnn_u, NULL, Dm, Dm, s, a, dtype);
    linear16(rnn_w, rnn_b, Dm, Dm, e, c, dtype);
    for (int i = 0; i < Dm; ++i) s_next[i] = silu(a[i] + c[i]);
    free(e);
    free(a);
    free(c);
}

void orc_draft(const uint16_t *emb, const uint16_t *rnn_u, const uint16_t *rnn_w, const float *rnn_b,
               const uint16_t *mlp_w, const float *mlp_b, int n_mlp, const uint16_t *head_w,
               const uint16_t *h /*[B][Dm]*/, const int32_t *last_token /*[B]*/,
               int B, int Dm, int V, int W, int L, int dtype /* ORC_BF16 or ORC_F16: weights, embeddings, h */,
               int32_t *beams /*[B][W][L]*/, float *beam_logp /*[B][W]*/,
               float *step_logp /*[L-1][B*W][V] or NULL*/, int32_t *step_row /*[B][W][L-1] or NULL*/)
{
    /* step_logp: the draft model's log-probabilities as they were computed during the search, row
     * b*W + w of step t-1 = live candidate w of sequence b at drafted position t (rows of candidates
     * that were not live, i.e. w >= 1 at the first position, are left untouched).  step_row[b][w][t-1]
     * = the row of step t-1 that produced token t of final candidate w, so that the draft
     * distribution behind every token of every candidate can be found without recomputation. */
    const int T = L - 1;
    int32_t *rows = (int32_t *)malloc(sizeof(int32_t) * (size_t)W * (T > 0 ? T : 1));
    int32_t *rows2 = (int32_t *)malloc(sizeof(int32_t) * (size_t)W * (T > 0 ? T : 1));
    double *hd = (double *)malloc(sizeof(double) * (size_t)Dm);
    double *s = (double *)malloc(sizeof(double) * (size_t)W * Dm);        /* state per live beam */
    double *s2 = (double *)malloc(sizeof(double) * (size_t)W * Dm);
    double *lp = (double *)malloc(sizeof(double) * (size_t)W * V);
    double *cum = (double *)malloc(sizeof(double) * (size_t)W), *cum2 = (double *)malloc(sizeof(double) * (size_t)W);
    int32_t *path = (int32_t *)malloc(sizeof(int32_t) * (size_t)W * L), *path2 = (int32_t *)malloc(sizeof(int32_t) * (size_t)W * L);
    unsigned char *taken = (unsigned char *)malloc((size_t)W * V);
    for (int b = 0; b < B; ++b) {
        for (int i = 0; i < Dm; ++i) {
            hd[i] = w16_to_double(h[(size_t)b * Dm + i], dtype);
            s[i] = w16_to_double(emb[(size_t)last_token[b] * Dm + i], dtype);
        }
        int live = 1;
        cum[0] = 0.0;
        path[0] = last_token[b];
        for (int w = 0; w < W; ++w) { beam_logp[(size_t)b * W + w] = 0.f; for (int j = 0; j < L; ++j) beams[((size_t)b * W + w) * L + j] = last_token[b]; }
        for (int t = 1; t <= T; ++t) {
            for (int w = 0; w < live; ++w)
                draft_logp(mlp_w, mlp_b, n_mlp, head_w, s + (size_t)w * Dm, hd, Dm, V, lp + (size_t)w * V, dtype);
            if (step_logp)
                for (int w = 0; w < live; ++w)
                    for (int v = 0; v < V; ++v)
                        step_logp[(((size_t)(t - 1) * B + b) * W + w) * V + v] = (float)lp[(size_t)w * V + v];
            memset(taken, 0, (size_t)live * V);
            for (int r = 0; r < W; ++r) {                 /* the r-th best candidate (beam w, token v) */
                int bw = -1, bv = -1;
                double best = -INFINITY;
                for (int w = 0; w < live; ++w)
                    for (int v = 0; v < V; ++v) {
                        if (taken[(size_t)w * V + v]) continue;
                        const double sc = cum[w] + lp[(size_t)w * V + v];
                        if (bw < 0 || sc > best) { best = sc; bw = w; bv = v; }   /* scan order = (w, v) ascending */
                    }
                taken[(size_t)bw * V + bv] = 1;
                cum2[r] = best;
                memcpy(path2 + (size_t)r * L, path + (size_t)bw * L, sizeof(int32_t) * (size_t)t);
                path2[(size_t)r * L + t] = bv;
                memcpy(rows2 + (size_t)r * T, rows + (size_t)bw * T, sizeof(int32_t) * (size_t)(t - 1));
                rows2[(size_t)r * T + t - 1] = b * W + bw;
                if (t < T) draft_rnn(emb, rnn_u, rnn_w, rnn_b, s + (size_t)bw * Dm, bv, Dm, s2 + (size_t)r * Dm, dtype);
            }
            live = W;
            memcpy(cum, cum2, sizeof(double) * (size_t)W);
            memcpy(path, path2, sizeof(int32_t) * (size_t)W * L);
            memcpy(rows, rows2, sizeof(int32_t) * (size_t)W * T);
            if (t < T) memcpy(s, s2, sizeof(double) * (size_t)W * Dm);
        }
        if (T >= 1)
            for (int w = 0; w < W; ++w) {
                beam_logp[(size_t)b * W + w] = (float)cum[w];
                memcpy(beams + ((size_t)b * W + w) * L, path + (size_t)w * L, sizeof(int32_t) * (size_t)L);
                if (step_row) memcpy(step_row + ((size_t)b * W + w) * T, rows + (size_t)w * T, sizeof(int32_t) * (size_t)T);
            }
    }
    free(rows); free(rows2);
    free(hd); free(s); free(s2); free(lp); free(cum); free(cum2); free(path); free(path2); free(taken);
}

/* Cumulative log probability of given candidates under the draft model (teacher forcing):
 * paths [B][n_paths][L] with position 0 the LLM's token; out [B][n_paths].               */
void orc_draft_path_logp(const uint16_t *emb, const uint16_t *rnn_u, const uint16_t *rnn_w, const float *rnn_b,
                         const uint16_t *mlp_w, const float *mlp_b, int n_mlp, const uint16_t *head_w,
                         const uint16_t *h, const int32_t *paths, int B, int n_paths, int Dm, int V, int L, int dtype,
                         double *out)
{
    double *hd = (double *)malloc(sizeof(double) * (size_t)Dm);
    double *s = (double *)malloc(sizeof(double) * (size_t)Dm), *s2 = (double *)malloc(sizeof(double) * (size_t)Dm);
    double *lp = (double *)malloc(sizeof(double) * (size_t)V);
    for (int b = 0; b < B; ++b)
        for (int r = 0; r < n_paths; ++r) {
            const int32_t *p = paths + ((size_t)b * n_paths + r) * L;
            for (int i = 0; i < Dm; ++i) {
                hd[i] = w16_to_double(h[(size_t)b * Dm + i], dtype);
                s[i] = w16_to_double(emb[(size_t)p[0] * Dm + i], dtype);
            }
            double total = 0.0;
            for (int t = 1; t < L; ++t) {
                draft_logp(mlp_w, mlp_b, n_mlp, head_w, s, hd, Dm, V, lp, dtype);
                total += lp[p[t]];
                if (t + 1 < L) {
                    draft_rnn(emb, rnn_u, rnn_w, rnn_b, s, p[t], Dm, s2, dtype);
                    memcpy(s, s2, sizeof(double) * (size_t)Dm);
                }
            }
            out[(size_t)b * n_paths + r] = total;
        }
    free(hd); free(s); free(s2); free(lp);
}

/* ---------------------------------------------------------------------------------
 * Acceptance by rejection sampling, the selection mode of Sec. 3.4 for sampling at a
 * temperature (the paper names the mode and gives no procedure; this is speculative
 * sampling as published by Leviathan et al. and Chen et al., 2023, applied to every
 * candidate of the beam on the packed tree).  Per sequence:
 *   p_s = softmax(logits[s] / temperature)   the LLM's distribution after packed token s
 *   q_s = softmax(draft_logits[s])           the draft model's distribution at the same place
 *   candidate w's token j >= 1 (x = beams[w][j], hanging under slot s = unpack[w][j-1], stored
 *   in slot c = unpack[w][j]) is accepted, given all earlier ones were, iff
 *       u_accept[c] < min(1, p_s(x) / q_s(x));
 *   the uniform number belongs to the packed slot, so candidates that share a prefix share
 *   its decisions.  Token 0 as in token matching (given, or compared with root_token).
 *   The best candidate has the longest accepted prefix (smallest index among equals).
 *   The token that follows it is drawn by inverting the cumulative distribution with
 *   u_next[b]: from p_s when the whole candidate was accepted, else from the residual
 *   max(0, p_s - q_s) (normalised) at the slot s under which its first rejected token hangs;
 *   it is the smallest v with  sum_{v' <= v} weight(v') > u_next * sum_v weight(v)  (the last
 *   v of positive weight if rounding leaves none).  A residual that vanishes identically
 *   (p_s == q_s) falls back to p_s.  With nothing accepted (root mismatch) the next token is
 *   root_token.
 * draft_logits rows of slots at the last position (depth L-1) are never read: the draft model
 * has no distribution there, and after a fully accepted candidate the LLM's own is used.
 * Diagnostics for the tests (each may be NULL): accept_ratio[b][w][j] = min(1, p/q) of every
 * token that was examined (j >= 1; -1 where the scan had already stopped), next_weights[b][v] =
 * the normalised distribution the next token was drawn from (zeros when best_len == 0).   */
static double log_sum_exp(const float *z, int V, double inv_t)
{
    double m = -INFINITY;
    for (int v = 0; v < V; ++v)
        if ((double)z[v] * inv_t > m) m = (double)z[v] * inv_t;
    if (m == -INFINITY) return m;
    double s = 0.0;
    for (int v = 0; v < V; ++v) s += exp((double)z[v] * inv_t - m);
    return m + log(s);
}

/* Where the draft model's logits of the distribution after candidate w's token j live: row
 * unpack_index[w][j] of the packed layout [B][N][V], or, when the rows recorded during the beam
 * search are handed over as they are (step layout [L-1][rows_per_step][V], step_row [B][W][L-1]),
 * row step_row[b][w][j] of step j.                                                          */
static const float *draft_row_of(const float *draft_logits, const int32_t *step_row, int rows_per_step,
                                 const int32_t *ui, int b, int w, int j, int W, int L, int V)
{
    const int N = W * L;
    if (step_row == NULL) return draft_logits + ((size_t)b * N + ui[w * L + j]) * V;
    return draft_logits + ((size_t)j * rows_per_step + step_row[((size_t)b * W + w) * (L - 1) + j]) * V;
}

void orc_accept_sample(const float *logits, const float *draft_logits, const int32_t *step_row, int rows_per_step,
                       const int32_t *beams, const int32_t *unpack_index, const int32_t *root_token,
                       const float *u_accept /*[B,N]*/, const float *u_next /*[B]*/, double temperature,
                       int B, int W, int L, int V,
                       int32_t *n_accept, int32_t *best_beam, int32_t *best_len, int32_t *next_token,
                       int32_t *accepted_idx, double *accept_ratio, double *next_weights)
{
    const int N = W * L;
    const double inv_t = 1.0 / temperature;
    double *wt = (double *)malloc(sizeof(double) * (size_t)V);
    for (int b = 0; b < B; ++b) {
        const int32_t *beam = beams + (size_t)b * N;
        const int32_t *ui = unpack_index + (size_t)b * N;
        int bw = 0, bl = -1;
        for (int w = 0; w < W; ++w) {
            int len = 0;
            if (accept_ratio)
                for (int j = 0; j < L; ++j) accept_ratio[((size_t)b * W + w) * L + j] = -1.0;
            for (int j = 0; j < L; ++j) {
                int ok;
                if (j == 0) {
                    ok = (root_token == NULL) || (beam[w * L] == root_token[b]);
                } else {
                    const int s = ui[w * L + j - 1], c = ui[w * L + j], x = beam[w * L + j];
                    const float *zp = logits + ((size_t)b * N + s) * V;
                    const float *zq = draft_row_of(draft_logits, step_row, rows_per_step, ui, b, w, j - 1, W, L, V);
                    double ratio = 0.0;                     /* a token outside the vocabulary is rejected */
                    if (x >= 0 && x < V) {
                        const double lp = (double)zp[x] * inv_t - log_sum_exp(zp, V, inv_t);
                        const double lq = (double)zq[x] - log_sum_exp(zq, V, 1.0);
                        ratio = exp(lp - lq);               /* p(x) / q(x) */
                        if (ratio > 1.0) ratio = 1.0;
                    }
                    if (accept_ratio) accept_ratio[((size_t)b * W + w) * L + j] = ratio;
                    ok = (double)u_accept[(size_t)b * N + c] < ratio;
                }
                if (!ok) break;
                ++len;
            }
            n_accept[b * W + w] = len;
            if (len > bl) { bl = len; bw = w; }
        }
        best_beam[b] = bw;
        best_len[b] = bl;
        for (int t = 0; t < L; ++t) accepted_idx[b * L + t] = (t < bl) ? ui[bw * L + t] : -1;
        if (next_weights) memset(next_weights + (size_t)b * V, 0, sizeof(double) * (size_t)V);
        if (bl == 0) {
            next_token[b] = root_token[b];
            continue;
        }
        const int s = ui[bw * L + bl - 1];
        const float *zp = logits + ((size_t)b * N + s) * V;
        const double lse_p = log_sum_exp(zp, V, inv_t);
        double total = 0.0;
        if (bl < L) {                                       /* a rejection: the residual distribution */
            const float *zq = draft_row_of(draft_logits, step_row, rows_per_step, ui, b, bw, bl - 1, W, L, V);
            const double lse_q = log_sum_exp(zq, V, 1.0);
            for (int v = 0; v < V; ++v) {
                const double d = exp((double)zp[v] * inv_t - lse_p) - exp((double)zq[v] - lse_q);
                wt[v] = d > 0.0 ? d : 0.0;
                total += wt[v];
            }
        }
        if (bl == L || total == 0.0) {
            total = 0.0;
            for (int v = 0; v < V; ++v) {
                wt[v] = exp((double)zp[v] * inv_t - lse_p);
                total += wt[v];
            }
        }
        const double target = (double)u_next[b] * total;
        int pick = -1, last_pos = 0;
        double cum = 0.0;
        for (int v = 0; v < V; ++v) {
            cum += wt[v];
            if (wt[v] > 0.0) last_pos = v;
            if (pick < 0 && cum > target) pick = v;
        }
        next_token[b] = pick >= 0 ? pick : last_pos;
        if (next_weights)
            for (int v = 0; v < V; ++v) next_weights[(size_t)b * V + v] = wt[v] / total;
    }
    free(wt);
}
