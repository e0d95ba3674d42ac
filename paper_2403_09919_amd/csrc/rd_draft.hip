// rd_draft: the draft model and its beam search (Sec. 3.1, 3.2) for gfx950.
//
// Per drafted position the work is three kinds of launches on the caller's stream:
//   * skinny linear layers  Y[M,N] = X[M,K] W[N,K]^T  with M = B*W rows (one per live candidate)
//     and bf16 weights streamed once from HBM: the layers are bound by that stream (the LM-head
//     alone is V x 2Dm), so a workgroup owns 16 output columns, its four waves split K, weights
//     go from memory straight into the A operand of v_mfma_f32_16x16x32_bf16 (lane = one output
//     column x 8 consecutive k), the activations (a few hundred KB, L2 resident) into the B
//     operand, and the four partial sums meet in LDS.  Bias, SiLU, skip connection and the bf16
//     copy that the next layer reads are fused into the epilogue;
//   * log-softmax over the vocabulary and the W best tokens of every row;
//   * the beam step: the best W of the (candidate, token) pairs of a sequence by cumulative log
//     probability, ties to the smaller candidate, then the smaller token.
// The RNN update reads its two inputs in place: the parent's state through a row map and the
// chosen token's embedding straight from the table, so no gather pass exists.
//
// Precision contract: weights, embeddings and h are bf16; every linear layer reads its input
// rounded to bf16 and accumulates in fp32; bias, activation, skip connection, log-softmax and
// scores are fp32.
#include "rd_internal.h"
#include <math.h>

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kLinThreads = 256;       // 4 waves: K is split four ways
constexpr int kMaxRows = 128;          // B*W
constexpr int kMaxBeam = 32;           // W
constexpr int kTopThreads = 1024;
constexpr int kTopPer = 32;            // logits per thread held in registers: V <= 32768

enum { EPI_HEAD = 0, EPI_RNN = 1, EPI_MLP = 2 };

struct LinArgs {
    // Y = X1 W1^T (+ X2 W2^T) + bias;  W row-major [N][K]; X rows found through row maps
    const __bf16 *w1, *w2;
    const __bf16 *x1, *x2;             // row r of X1 is x1 + map1[r]*ldx1 (map NULL: r itself)
    const int32_t *map1, *map2;
    int ldx1, ldx2, K1, K2;            // K2 = 0: single product
    const float *bias;                 // [N] or NULL
    int M, N;
    // epilogue
    float *y_f32;                      // HEAD: logits [M][ldy];  RNN/MLP: activations fp32 [M][ldy]
    __bf16 *y_bf;                      // RNN/MLP: the same rounded to bf16 [M][ldy]
    __bf16 *s_bf;                      // RNN: next state [M][N]
    const float *res;                  // MLP: skip input fp32 [M][ldy]
    int ldy;
};

__device__ __forceinline__ float silu(float x) { return x / (1.0f + __expf(-x)); }

template <int MT, int EPI>
__global__ __launch_bounds__(kLinThreads) void rd_linear_kernel(LinArgs a)
{
    __shared__ f32x4 s_part[3][MT][64];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r16 = lane & 15, g = lane >> 4;
    const int n0 = blockIdx.x * 16;

    // this wave's share of the k-steps (32 wide); the host guarantees it lies within one product
    const int ks1 = a.K1 >> 5, ks = ks1 + (a.K2 >> 5);
    const int kb = (int)((long long)ks * wave / 4), ke = (int)((long long)ks * (wave + 1) / 4);
    const bool second = kb >= ks1;
    const __bf16 *wbase = second ? a.w2 : a.w1;
    const int K = second ? a.K2 : a.K1;
    const int k_first = (second ? kb - ks1 : kb) * 32, steps = ke - kb;
    const __bf16 *xbase = second ? a.x2 : a.x1;
    const int32_t *map = second ? a.map2 : a.map1;
    const int ldx = second ? a.ldx2 : a.ldx1;

    const int nrow = min(n0 + r16, a.N - 1);                    // rows past N read the last row; never stored
    const __bf16 *wp = wbase + (size_t)nrow * K + k_first + 8 * g;
    const __bf16 *xp[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int m = min(mt * 16 + r16, a.M - 1);
        const int row = map ? map[m] : m;
        xp[mt] = xbase + (size_t)row * ldx + k_first + 8 * g;
    }
    f32x4 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};

    constexpr int U = 4;                                        // k-steps in flight
    int s = 0;
    for (; s + U <= steps; s += U) {
        bf16x8 wa[U], xb[U][MT];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            wa[u] = *reinterpret_cast<const bf16x8 *>(wp + (s + u) * 32);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) xb[u][mt] = *reinterpret_cast<const bf16x8 *>(xp[mt] + (s + u) * 32);
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa[u], xb[u][mt], acc[mt], 0, 0, 0);
    }
    for (; s < steps; ++s) {
        const bf16x8 wa = *reinterpret_cast<const bf16x8 *>(wp + s * 32);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const bf16x8 xb = *reinterpret_cast<const bf16x8 *>(xp[mt] + s * 32);
            acc[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa, xb, acc[mt], 0, 0, 0);
        }
    }

    // the four K-quarters meet in LDS; wave 0 finishes
    if (wave > 0) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) s_part[wave - 1][mt][lane] = acc[mt];
    }
    __syncthreads();
    if (wave > 0) return;
    // accumulator layout: element i of lane (r16, g) is output column n0 + 4g + i of row mt*16 + r16
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        f32x4 v = acc[mt] + s_part[0][mt][lane] + s_part[1][mt][lane] + s_part[2][mt][lane];
        const int m = mt * 16 + r16;
        if (m >= a.M) continue;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int n = n0 + 4 * g + i;
            if (n >= a.N) continue;
            float y = v[i] + (a.bias ? a.bias[n] : 0.f);
            const size_t o = (size_t)m * a.ldy + n;
            if (EPI == EPI_HEAD) {
                a.y_f32[o] = y;
            } else {
                y = silu(y);
                if (EPI == EPI_MLP) y += a.res[o];
                a.y_f32[o] = y;
                a.y_bf[o] = (__bf16)y;
                if (EPI == EPI_RNN) a.s_bf[(size_t)m * a.N + n] = (__bf16)y;
            }
        }
    }
}

// rows m = b*W + w: X0 = [e(last token), h] (fp32 and bf16), state = e(last token), path = [last token]
__global__ void rd_draft_init_kernel(const __bf16 *__restrict__ emb, const __bf16 *__restrict__ h,
                                     const int32_t *__restrict__ last_token, int W, int L, int Dm, int V,
                                     float *__restrict__ x_f32, __bf16 *__restrict__ x_bf, __bf16 *__restrict__ s_bf,
                                     int32_t *__restrict__ paths, float *__restrict__ cum)
{
    const int m = blockIdx.x, b = m / W;
    int tok = last_token[b];
    tok = tok < 0 ? 0 : (tok > V - 1 ? V - 1 : tok);
    for (int i = threadIdx.x; i < Dm; i += blockDim.x) {
        const __bf16 e = emb[(size_t)tok * Dm + i], hv = h[(size_t)b * Dm + i];
        x_f32[(size_t)m * 2 * Dm + i] = (float)e;
        x_bf[(size_t)m * 2 * Dm + i] = e;
        x_f32[(size_t)m * 2 * Dm + Dm + i] = (float)hv;
        x_bf[(size_t)m * 2 * Dm + Dm + i] = hv;
        s_bf[(size_t)m * Dm + i] = e;
    }
    for (int j = threadIdx.x; j < L; j += blockDim.x) paths[(size_t)m * L + j] = tok;
    if (threadIdx.x == 0) cum[m] = 0.f;
}

__device__ __forceinline__ bool better(float v, int i, float bv, int bi) { return v > bv || (v == bv && i < bi); }

// One workgroup per row: log-softmax over V logits and the W best tokens (value first, then the
// smaller index), as cumulative scores cand_score[m][r] = cum[m] + log p and tokens cand_tok[m][r].
__global__ __launch_bounds__(kTopThreads) void rd_topw_kernel(const float *__restrict__ logits, int V, int W,
                                                              const float *__restrict__ cum,
                                                              float *__restrict__ cand_score, int32_t *__restrict__ cand_tok)
{
    __shared__ float s_v[kTopThreads / 64];
    __shared__ int s_i[kTopThreads / 64];
    __shared__ float s_bcast[2];
    __shared__ int s_win;
    const int m = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float *z = logits + (size_t)m * V;
    float x[kTopPer];
    float mx = -INFINITY;
#pragma unroll
    for (int j = 0; j < kTopPer; ++j) {
        const int v = j * kTopThreads + tid;
        x[j] = v < V ? z[v] : -INFINITY;
        mx = fmaxf(mx, x[j]);
    }
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
    if (lane == 0) s_v[wave] = mx;
    __syncthreads();
    if (tid == 0) {
        float t = s_v[0];
        for (int w = 1; w < kTopThreads / 64; ++w) t = fmaxf(t, s_v[w]);
        s_bcast[0] = t;
    }
    __syncthreads();
    mx = s_bcast[0];
    float sum = 0.f;
#pragma unroll
    for (int j = 0; j < kTopPer; ++j) sum += (j * kTopThreads + tid < V) ? __expf(x[j] - mx) : 0.f;
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, 64);
    __syncthreads();
    if (lane == 0) s_v[wave] = sum;
    __syncthreads();
    if (tid == 0) {
        float t = 0.f;
        for (int w = 0; w < kTopThreads / 64; ++w) t += s_v[w];
        s_bcast[1] = mx + __logf(t);
    }
    __syncthreads();
    const float lse = s_bcast[1];
    const float base = cum[m];

    uint32_t gone = 0;                          // bit j: x[j] already taken
    float lv = -INFINITY;                       // this thread's best remaining (value, index)
    int li = 0x7fffffff;
    bool stale = true;
    for (int r = 0; r < W; ++r) {
        if (stale) {
            lv = -INFINITY;
            li = 0x7fffffff;
#pragma unroll
            for (int j = 0; j < kTopPer; ++j) {
                const int v = j * kTopThreads + tid;
                if (v < V && !((gone >> j) & 1u) && better(x[j], v, lv, li)) { lv = x[j]; li = v; }
            }
            stale = false;
        }
        float bv = lv;
        int bi = li;
        for (int off = 32; off > 0; off >>= 1) {
            const float ov = __shfl_xor(bv, off, 64);
            const int oi = __shfl_xor(bi, off, 64);
            if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
        }
        __syncthreads();
        if (lane == 0) { s_v[wave] = bv; s_i[wave] = bi; }
        __syncthreads();
        if (tid == 0) {
            for (int w = 1; w < kTopThreads / 64; ++w)
                if (better(s_v[w], s_i[w], bv, bi)) { bv = s_v[w]; bi = s_i[w]; }
            s_win = bi;
            cand_score[(size_t)m * W + r] = base + (bv - lse);
            cand_tok[(size_t)m * W + r] = bi;
        }
        __syncthreads();
        const int win = s_win;
        if (win == li) {                         // mine: retire it
            gone |= 1u << (win / kTopThreads);
            stale = true;
        }
    }
}

// One workgroup per sequence: the best W of live*W candidates (live = 1 at the first position).
// Candidate c = w*W + r (row w's r-th best token); ties in score go to the smaller c, which is
// the smaller candidate first and, within a row, the smaller token (rows are sorted that way).
__global__ __launch_bounds__(256) void rd_beam_select_kernel(
    const float *__restrict__ cand_score, const int32_t *__restrict__ cand_tok, int W, int L, int t, int live,
    const int32_t *__restrict__ paths_cur, int32_t *__restrict__ paths_next, float *__restrict__ cum_next,
    int32_t *__restrict__ parent_row, int32_t *__restrict__ tok_row,
    int32_t *__restrict__ beams_out, float *__restrict__ logp_out /* both NULL except at the last position */)
{
    __shared__ float s_v[4];
    __shared__ int s_i[4];
    __shared__ int s_win;
    __shared__ float s_winv;
    constexpr int kPer = (kMaxBeam * kMaxBeam + 255) / 256;
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n_cand = live * W;
    float x[kPer];
#pragma unroll
    for (int j = 0; j < kPer; ++j) {
        const int c = j * 256 + tid;
        x[j] = c < n_cand ? cand_score[(size_t)b * W * W + c] : -INFINITY;     // rows of sequence b are contiguous
    }
    uint32_t gone = 0;
    for (int r = 0; r < W; ++r) {
        float bv = -INFINITY;
        int bi = 0x7fffffff;
#pragma unroll
        for (int j = 0; j < kPer; ++j) {
            const int c = j * 256 + tid;
            if (c < n_cand && !((gone >> j) & 1u) && better(x[j], c, bv, bi)) { bv = x[j]; bi = c; }
        }
        for (int off = 32; off > 0; off >>= 1) {
            const float ov = __shfl_xor(bv, off, 64);
            const int oi = __shfl_xor(bi, off, 64);
            if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
        }
        __syncthreads();
        if (lane == 0) { s_v[wave] = bv; s_i[wave] = bi; }
        __syncthreads();
        if (tid == 0) {
            for (int w = 1; w < 4; ++w)
                if (better(s_v[w], s_i[w], bv, bi)) { bv = s_v[w]; bi = s_i[w]; }
            s_win = bi;
            s_winv = bv;
        }
        __syncthreads();
        const int win = s_win;
        if ((win & 255) == tid) gone |= 1u << (win >> 8);
        const int pw = win / W;                                   // parent candidate
        const int tok = cand_tok[(size_t)b * W * W + win];
        const size_t dst = ((size_t)b * W + r) * L, src = ((size_t)b * W + pw) * L;
        for (int j = tid; j < L; j += 256) {
            const int v = j < t ? paths_cur[src + j] : (j == t ? tok : paths_cur[src]);
            paths_next[dst + j] = v;
            if (beams_out) beams_out[dst + j] = v;
        }
        if (tid == 0) {
            cum_next[(size_t)b * W + r] = s_winv;
            parent_row[(size_t)b * W + r] = b * W + pw;
            tok_row[(size_t)b * W + r] = tok;
            if (logp_out) logp_out[(size_t)b * W + r] = s_winv;
        }
    }
}

struct Plan {
    size_t x_f32[3], x_bf[3], s_bf[2], logits, cand_score, cand_tok, paths[2], cum[2], parent, tok, total;
};

Plan draft_plan(int B, int W, int L, int Dm, int V)
{
    Plan p;
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t o = off; off += (bytes + 255) / 256 * 256; return o; };
    const size_t M = (size_t)B * W, G = 2 * (size_t)Dm;
    for (int i = 0; i < 3; ++i) { p.x_f32[i] = take(M * G * 4); p.x_bf[i] = take(M * G * 2); }
    for (int i = 0; i < 2; ++i) p.s_bf[i] = take(M * Dm * 2);
    p.logits = take(M * (size_t)V * 4);
    p.cand_score = take(M * W * 4);
    p.cand_tok = take(M * W * 4);
    for (int i = 0; i < 2; ++i) { p.paths[i] = take(M * L * 4); p.cum[i] = take(M * 4); }
    p.parent = take(M * 4);
    p.tok = take(M * 4);
    p.total = off;
    return p;
}

int draft_check(const rd_draft_params *p, int B, int W, int L)
{
    if (!p || B <= 0 || W <= 0 || L <= 0) return RD_ERR_INVALID_ARG;
    if (p->Dm <= 0 || p->V <= 0 || p->n_mlp < 0) return RD_ERR_INVALID_ARG;
    if (p->Dm % 64 != 0) return RD_ERR_UNSUPPORTED;              // every wave's K share is whole 32-wide steps
    if (W > kMaxBeam || (long long)B * W > kMaxRows || W > p->V) return RD_ERR_UNSUPPORTED;
    if (p->V > kTopThreads * kTopPer || L > RD_MAX_N) return RD_ERR_UNSUPPORTED;
    return RD_OK;
}

template <int EPI>
int launch_linear(const LinArgs &a, hipStream_t stream)
{
    const dim3 grid((a.N + 15) / 16), block(kLinThreads);
    const int mt = (a.M + 15) / 16;
    if (mt <= 1) hipLaunchKernelGGL((rd_linear_kernel<1, EPI>), grid, block, 0, stream, a);
    else if (mt <= 2) hipLaunchKernelGGL((rd_linear_kernel<2, EPI>), grid, block, 0, stream, a);
    else if (mt <= 4) hipLaunchKernelGGL((rd_linear_kernel<4, EPI>), grid, block, 0, stream, a);
    else hipLaunchKernelGGL((rd_linear_kernel<8, EPI>), grid, block, 0, stream, a);
    return rd_check_launch();
}

}  // namespace

extern "C" size_t rd_draft_workspace(int B, int W, int L, int Dm, int V)
{
    rd_draft_params p = {};
    p.Dm = Dm; p.V = V;
    if (draft_check(&p, B, W, L) != RD_OK) return 0;
    return draft_plan(B, W, L, Dm, V).total;
}

extern "C" int rd_draft(const rd_draft_params *p, const void *h, const int32_t *last_token,
                        int B, int W, int L, int32_t *beams, float *beam_logp,
                        void *workspace, size_t workspace_bytes, void *stream)
{
    const int st = draft_check(p, B, W, L);
    if (st != RD_OK) return st;
    if (!p->emb || !p->rnn_u || !p->rnn_w || !p->rnn_b || !p->head_w || (p->n_mlp > 0 && (!p->mlp_w || !p->mlp_b)))
        return RD_ERR_INVALID_ARG;
    if (!h || !last_token || !beams || !beam_logp) return RD_ERR_INVALID_ARG;
    if (!rd_aligned(p->emb, 16) || !rd_aligned(p->rnn_u, 16) || !rd_aligned(p->rnn_w, 16) || !rd_aligned(p->mlp_w, 16) ||
        !rd_aligned(p->head_w, 16) || !rd_aligned(h, 16))
        return RD_ERR_INVALID_ARG;
    const Plan plan = draft_plan(B, W, L, p->Dm, p->V);
    if (!workspace || !rd_aligned(workspace, 256) || workspace_bytes < plan.total) return RD_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    unsigned char *ws = static_cast<unsigned char *>(workspace);
    const int Dm = p->Dm, G = 2 * Dm, V = p->V, M = B * W, T = L - 1;
    float *x_f32[3];
    __bf16 *x_bf[3], *s_bf[2];
    for (int i = 0; i < 3; ++i) { x_f32[i] = reinterpret_cast<float *>(ws + plan.x_f32[i]); x_bf[i] = reinterpret_cast<__bf16 *>(ws + plan.x_bf[i]); }
    for (int i = 0; i < 2; ++i) s_bf[i] = reinterpret_cast<__bf16 *>(ws + plan.s_bf[i]);
    float *logits = reinterpret_cast<float *>(ws + plan.logits);
    float *cand_score = reinterpret_cast<float *>(ws + plan.cand_score);
    int32_t *cand_tok = reinterpret_cast<int32_t *>(ws + plan.cand_tok);
    int32_t *paths[2] = {reinterpret_cast<int32_t *>(ws + plan.paths[0]), reinterpret_cast<int32_t *>(ws + plan.paths[1])};
    float *cum[2] = {reinterpret_cast<float *>(ws + plan.cum[0]), reinterpret_cast<float *>(ws + plan.cum[1])};
    int32_t *parent = reinterpret_cast<int32_t *>(ws + plan.parent), *tok = reinterpret_cast<int32_t *>(ws + plan.tok);
    const __bf16 *emb = static_cast<const __bf16 *>(p->emb);

    hipLaunchKernelGGL(rd_draft_init_kernel, dim3(M), dim3(256), 0, s, emb, static_cast<const __bf16 *>(h), last_token,
                       W, L, Dm, V, x_f32[0], x_bf[0], s_bf[0], paths[0], cum[0]);
    if (rd_check_launch() != RD_OK) return RD_ERR_HIP;
    if (T == 0) {                                   // nothing to draft: the candidates are the LLM's token alone
        hipLaunchKernelGGL(rd_draft_init_kernel, dim3(M), dim3(256), 0, s, emb, static_cast<const __bf16 *>(h), last_token,
                           W, L, Dm, V, x_f32[0], x_bf[0], s_bf[0], beams, beam_logp);
        return rd_check_launch();
    }
    // the h half of X0 must survive the MLP ping-pong: layers write X1 and X2 only
    int si = 0;                                     // state buffer holding s_t of the live candidates
    for (int t = 1; t <= T; ++t) {
        const int cur = (t - 1) & 1, nxt = t & 1;
        if (t > 1) {                                // s_t = f(U s_{t-1}[parent] + W e(token) + b) -> X0[:, :Dm]
            LinArgs a = {};
            a.w1 = static_cast<const __bf16 *>(p->rnn_u); a.x1 = s_bf[si]; a.map1 = parent; a.ldx1 = Dm; a.K1 = Dm;
            a.w2 = static_cast<const __bf16 *>(p->rnn_w); a.x2 = emb; a.map2 = tok; a.ldx2 = Dm; a.K2 = Dm;
            a.bias = p->rnn_b; a.M = M; a.N = Dm;
            a.y_f32 = x_f32[0]; a.y_bf = x_bf[0]; a.s_bf = s_bf[si ^ 1]; a.ldy = G;
            if (launch_linear<EPI_RNN>(a, s) != RD_OK) return RD_ERR_HIP;
            si ^= 1;
        }
        int in = 0;
        for (int k = 0; k < p->n_mlp; ++k) {        // x <- x + f(A_k x + c_k)
            const int out = in == 1 ? 2 : 1;
            LinArgs a = {};
            a.w1 = static_cast<const __bf16 *>(p->mlp_w) + (size_t)k * G * G; a.x1 = x_bf[in]; a.ldx1 = G; a.K1 = G;
            a.bias = p->mlp_b + (size_t)k * G; a.M = M; a.N = G;
            a.y_f32 = x_f32[out]; a.y_bf = x_bf[out]; a.res = x_f32[in]; a.ldy = G;
            if (launch_linear<EPI_MLP>(a, s) != RD_OK) return RD_ERR_HIP;
            in = out;
        }
        {                                           // logits
            LinArgs a = {};
            a.w1 = static_cast<const __bf16 *>(p->head_w); a.x1 = x_bf[in]; a.ldx1 = G; a.K1 = G;
            a.M = M; a.N = V; a.y_f32 = logits; a.ldy = V;
            if (launch_linear<EPI_HEAD>(a, s) != RD_OK) return RD_ERR_HIP;
        }
        hipLaunchKernelGGL(rd_topw_kernel, dim3(M), dim3(kTopThreads), 0, s, logits, V, W, cum[cur], cand_score, cand_tok);
        if (rd_check_launch() != RD_OK) return RD_ERR_HIP;
        const bool last = t == T;
        hipLaunchKernelGGL(rd_beam_select_kernel, dim3(B), dim3(256), 0, s, cand_score, cand_tok, W, L, t, t == 1 ? 1 : W,
                           paths[cur], paths[nxt], cum[nxt], parent, tok, last ? beams : nullptr, last ? beam_logp : nullptr);
        if (rd_check_launch() != RD_OK) return RD_ERR_HIP;
    }
    return RD_OK;
}
