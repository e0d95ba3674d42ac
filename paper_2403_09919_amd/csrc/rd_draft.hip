// rd_draft: the draft model and its beam search (Sec. 3.1, 3.2) for gfx950.
//
// Per drafted position the work is two kinds of launches on the caller's stream:
//   * skinny linear layers  Y[M,N] = X[M,K] W[N,K]^T  with M = B*W rows (one per live candidate)
//     and bf16 weights streamed once from HBM: the layers are bound by that stream (the LM-head
//     alone is V x 2Dm), so a workgroup owns 16 to 64 output columns, its waves split K, weights
//     go from memory straight into the A operand of v_mfma_f32_16x16x32_bf16 (lane = one output
//     column x 8 consecutive k), the activations (a few hundred KB, L2 resident) into the B
//     operand, and the partial sums meet in LDS.  Bias, SiLU, skip connection and the bf16
//     copy that the next layer reads are fused into the epilogue.  At more than 32 rows the
//     layers with few columns use 128- or 64-column workgroups and split K over 2 to 8
//     workgroups per column group as well; the last of them to finish adds the partial tiles;
//   * three selection launches, all merges of sorted lists: per chunk of 4096 logits and row, the
//     pieces of the log-sum-exp and the W best tokens; per row, its log-sum-exp and the W best
//     tokens of its chunks as cumulative scores; per sequence, the best W of the (candidate, token)
//     pairs by cumulative log probability, ties to the smaller candidate, then the smaller token
//     (W <= 128; beyond 64 candidates a lane of the last merge holds two lists).
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
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;

// The 16-bit storage type of the model (bf16 or fp16): eight-element vector and its MFMA.
template <typename T> struct Elem16;
template <> struct Elem16<__bf16> {
    typedef bf16x8 vec8;
    static __device__ __forceinline__ f32x4 mfma(vec8 a, vec8 b, f32x4 c) { return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0); }
};
template <> struct Elem16<_Float16> {
    typedef f16x8 vec8;
    static __device__ __forceinline__ f32x4 mfma(vec8 a, vec8 b, f32x4 c) { return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0); }
};

constexpr int kMaxRows = 512;          // B*W
constexpr int kRowsPerLaunch = 128;    // rows of one linear-layer launch (8 MFMA row tiles)
constexpr int kMaxBeam = 128;          // W
constexpr int kNarrowBeam = 64;        // up to here the selection kernels keep their lists in static LDS, one candidate per lane
constexpr int kSelThreads = 256;       // row pass and beam step: four waves bring the lists into LDS, the first one merges
constexpr int kMaxVocab = 262144;      // 64 chunks of 4096 logits: one lane per chunk in the row pass
constexpr int kSplitMaxWgs = 256;      // workgroups of a launch whose K is split over workgroups
constexpr int kSplitMaxGroups = 128;   // ... and its column groups (one arrival counter each)
constexpr int kSplitTiles = 64;        // ... and the 16x16 output tiles a workgroup holds

enum { EPI_HEAD = 0, EPI_RNN = 1, EPI_MLP = 2 };

template <typename T>
struct LinArgs {
    // Y = X1 W1^T (+ X2 W2^T) + bias;  W row-major [N][K]; X rows found through row maps
    const T *w1, *w2;
    const T *x1, *x2;             // row r of X1 is x1 + map1[r]*ldx1 (map NULL: r itself)
    const int32_t *map1, *map2;
    int ldx1, ldx2, K1, K2;            // K2 = 0: single product
    int tiled;                         // weights in the operand-tiled layout of rd_draft_pack_weights
    const float *bias;                 // [N] or NULL
    int M, N;
    int m0;                            // first logical row of this launch (a launch covers rows m0 .. m0+M-1)
    int mstride;                       // logical row m of X (without a map), Y and res is physical row m*mstride
    // epilogue
    float *y_f32;                      // HEAD: logits [M][ldy];  RNN/MLP: activations fp32 [M][ldy]
    T *y_bf;                           // RNN/MLP: the same rounded to the storage type [M][ldy]
    T *s_bf;                           // RNN: next state [M][N]
    const float *res;                  // MLP: skip input fp32 [M][ldy]
    int ldy;
    // K split over workgroups (kernels instantiated with KSP): workgroup = (column group, split)
    int ksplit;                        // splits per column group
    float *kpart;                      // partial tiles [group][split][tile][64 lanes] x 4 floats
    uint32_t *kcount;                  // arrivals per column group, zero between launches
};

__device__ __forceinline__ float silu(float x) { return x / (1.0f + __expf(-x)); }

// One output tile (16 rows x 16 columns) leaves the kernel: bias, activation, skip connection and the
// bf16 copy that the next layer reads.  Accumulator layout: element i of lane (r16, g) is output
// column n_tile + 4g + i of logical row m_tile + r16.
template <typename T, int EPI>
__device__ __forceinline__ void linear_epilogue(const LinArgs<T> &a, f32x4 v, int m_tile, int n_tile, int r16, int g)
{
    const int m = m_tile + r16;
    if (m >= a.M) return;
    const size_t prow = (size_t)(a.m0 + m) * a.mstride;         // physical row of the activation buffers
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int n = n_tile + 4 * g + i;
        if (n >= a.N) continue;
        float y = v[i] + (a.bias ? a.bias[n] : 0.f);
        const size_t o = prow * a.ldy + n;
        if (EPI == EPI_HEAD) {
            a.y_f32[o] = y;
        } else {
            y = silu(y);
            if (EPI == EPI_MLP) y += a.res[o];
            a.y_f32[o] = y;
            a.y_bf[o] = (T)y;
            if (EPI == EPI_RNN) a.s_bf[prow * a.N + n] = (T)y;
        }
    }
}

// The last workgroup of a column group adds the KS partial tiles of each output tile in split order
// and finishes them.  A wave's loads are issued together (in batches of at most 32 partial tiles) before
// the sums.
template <typename T, int MT, int NT, int NWV, int EPI, int KS>
__device__ __forceinline__ void linear_finish_split(const LinArgs<T> &a, int group, int n0, int wave, int lane)
{
    constexpr int kTiles = MT * NT, kMine = kTiles / NWV;       // tiles per wave
    constexpr int kBatch = kMine * KS > 32 ? 32 / KS : kMine;   // tiles whose loads are in flight together (<= 128 registers)
    static_assert(kTiles % NWV == 0 && kMine % kBatch == 0, "every wave finishes the same number of tiles, in whole batches");
    const int r16 = lane & 15, g = lane >> 4;
#pragma unroll
    for (int i0 = 0; i0 < kMine; i0 += kBatch) {
        float2 lo[kBatch][KS], hi[kBatch][KS];
#pragma unroll
        for (int i = 0; i < kBatch; ++i)
#pragma unroll
            for (int sp = 0; sp < KS; ++sp) {
                const float *src = a.kpart + ((((size_t)group * KS + sp) * kTiles + wave + (i0 + i) * NWV) * 64 + lane) * 4;
                lo[i][sp] = rd::ld_dev2(src);
                hi[i][sp] = rd::ld_dev2(src + 2);
            }
#pragma unroll
        for (int i = 0; i < kBatch; ++i) {
            const int id = wave + (i0 + i) * NWV;
            f32x4 v = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int sp = 0; sp < KS; ++sp) v += f32x4{lo[i][sp].x, lo[i][sp].y, hi[i][sp].x, hi[i][sp].y};
            linear_epilogue<T, EPI>(a, v, (id / NT) * 16, n0 + (id % NT) * 16, r16, g);
        }
    }
}

// A workgroup owns NT*16 output columns for all M = MT*16 rows; its NWV waves split K.  The host
// picks NT so that the activations, which every workgroup re-reads through the caches, do not
// outweigh the weights it streams (their ratio is MT : NT) while the launch still covers the chip,
// and NWV so that the launch has enough waves in flight to keep the HBM stream busy; every wave's
// share of K is a whole number of 32-wide steps inside one of the two products.
//
// KSP: K is also split over a.ksplit workgroups per column group, for layers with so few columns that
// NT-wide workgroups alone would leave most of the chip idle.  Every workgroup stores its partial
// tiles (write-through) and signals; the last to arrive for its column group adds the partials in
// split order (so the sum does not depend on who was last) and runs the epilogue.
template <typename T, int MT, int NT, int NWV, int EPI, bool TILED, bool KSP = false>
__global__ __launch_bounds__(NWV * 64) void rd_linear_kernel(LinArgs<T> a)
{
    typedef typename Elem16<T>::vec8 vec8;
    constexpr int kTiles = MT * NT;
    constexpr int kGroup = kTiles < 64 / NWV ? kTiles : 64 / NWV;     // tiles reduced per pass: <= 64 KB of LDS
    static_assert(kTiles % kGroup == 0, "tile groups must divide the tiles");
    __shared__ f32x4 s_part[NWV][kGroup][64];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r16 = lane & 15, g = lane >> 4;
    const int groups = KSP ? (int)gridDim.x / a.ksplit : (int)gridDim.x;
    const int group = KSP ? (int)blockIdx.x % groups : (int)blockIdx.x;
    const int split = KSP ? (int)blockIdx.x / groups : 0;
    const int n0 = group * (16 * NT);

    // this wave's share of the k-steps (32 wide); the host guarantees it lies within one product
    const int ks1 = a.K1 >> 5, ks = ks1 + (a.K2 >> 5);
    const int parts = KSP ? a.ksplit * NWV : NWV, part = split * NWV + wave;
    const int kb = (int)((long long)ks * part / parts), ke = (int)((long long)ks * (part + 1) / parts);
    const bool second = kb >= ks1;
    const T *wbase = second ? a.w2 : a.w1;
    const int K = second ? a.K2 : a.K1;
    const int k_first = (second ? kb - ks1 : kb) * 32, steps = ke - kb;
    const T *xbase = second ? a.x2 : a.x1;
    const int32_t *map = second ? a.map2 : a.map1;
    const int ldx = second ? a.ldx2 : a.ldx1;

    const T *wp[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        if (TILED) {                                            // tile (n/16, k/32): 64 lanes x 8 elements, contiguous
            const int ntile = min(n0 / 16 + nt, (a.N + 15) / 16 - 1);
            wp[nt] = wbase + ((size_t)ntile * (K >> 5) + (k_first >> 5)) * 512 + lane * 8;
        } else {
            const int nrow = min(n0 + nt * 16 + r16, a.N - 1);  // rows past N read the last row; never stored
            wp[nt] = wbase + (size_t)nrow * K + k_first + 8 * g;
        }
    }
    const T *xp[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        const int m = a.m0 + min(mt * 16 + r16, a.M - 1);
        const size_t row = map ? (size_t)map[m] : (size_t)m * a.mstride;
        xp[mt] = xbase + row * ldx + k_first + 8 * g;
    }
    constexpr int wstep = TILED ? 512 : 32;                     // elements between a lane's vectors of consecutive k-steps
    f32x4 acc[MT][NT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[mt][nt] = f32x4{0.f, 0.f, 0.f, 0.f};

    constexpr int U = MT + NT <= 3 ? 8 : (MT + NT <= 9 ? 4 : 2);   // k-steps in flight
    int s = 0;
    for (; s + U <= steps; s += U) {
        vec8 wa[U][NT], xb[U][MT];
#pragma unroll
        for (int u = 0; u < U; ++u) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) wa[u][nt] = *reinterpret_cast<const vec8 *>(wp[nt] + (s + u) * wstep);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) xb[u][mt] = *reinterpret_cast<const vec8 *>(xp[mt] + (s + u) * 32);
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    acc[mt][nt] = Elem16<T>::mfma(wa[u][nt], xb[u][mt], acc[mt][nt]);
    }
    for (; s < steps; ++s) {
        vec8 wa[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) wa[nt] = *reinterpret_cast<const vec8 *>(wp[nt] + s * wstep);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            const vec8 xb = *reinterpret_cast<const vec8 *>(xp[mt] + s * 32);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                acc[mt][nt] = Elem16<T>::mfma(wa[nt], xb, acc[mt][nt]);
        }
    }

    // the K shares meet in LDS, a group of tiles at a time; tile j of a group is summed (in wave
    // order, so the result does not depend on timing) and finished by wave j mod NWV
#pragma unroll
    for (int p = 0; p < kTiles / kGroup; ++p) {
        if (p > 0) __syncthreads();
#pragma unroll
        for (int j = 0; j < kGroup; ++j) s_part[wave][j][lane] = acc[(p * kGroup + j) / NT][(p * kGroup + j) % NT];
        __syncthreads();
        for (int j = wave; j < kGroup; j += NWV) {
            f32x4 v = s_part[0][j][lane];
#pragma unroll
            for (int w = 1; w < NWV; ++w) v += s_part[w][j][lane];
            const int id = p * kGroup + j;
            if constexpr (KSP)
                rd::st_dev4(a.kpart + ((((size_t)group * a.ksplit + split) * kTiles + id) * 64 + lane) * 4, v[0], v[1], v[2], v[3]);
            else
                linear_epilogue<T, EPI>(a, v, (id / NT) * 16, n0 + (id % NT) * 16, r16, g);
        }
    }
    if constexpr (KSP) {
        __shared__ uint32_t s_last;
        rd::wait_dev_stores();
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");      // this workgroup's partial tiles are acknowledged
        __syncthreads();
        if (tid == 0) {
            const uint32_t prev = __hip_atomic_fetch_add(a.kcount + group, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            s_last = (prev + 1u == (uint32_t)a.ksplit) ? 1u : 0u;
            if (s_last) a.kcount[group] = 0;                        // ready for the next launch
        }
        __syncthreads();
        if (!s_last) return;
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
        if (a.ksplit == 8) linear_finish_split<T, MT, NT, NWV, EPI, 8>(a, group, n0, wave, lane);
        else if (a.ksplit == 4) linear_finish_split<T, MT, NT, NWV, EPI, 4>(a, group, n0, wave, lane);
        else linear_finish_split<T, MT, NT, NWV, EPI, 2>(a, group, n0, wave, lane);
    }
}

// The output layer at more than a few rows: with K split over the waves, the accumulators of 128 rows leave
// a workgroup room for only 64 columns, and every workgroup then pulls two activation bytes through the
// caches per weight byte (one per weight byte already at 16 rows, with 16-column workgroups).  Here the waves split the columns instead: a wave owns 32 columns for
// all rows (16 accumulator tiles) and half of every chunk's k-steps, so a workgroup of 8 waves covers 128
// columns with half of the registers (every B operand read from LDS feeds two matrix instructions), all
// waves walk K together in chunks of 256, and the activations of a chunk are staged once per
// workgroup in LDS (row stride 528 bytes: the 16 rows a B-operand read touches fall in distinct banks),
// double-buffered, one barrier per chunk.  Weights still go from memory straight into the A operand, one
// chunk ahead.  An output is the sum of two accumulators, each over its k-steps in order, for either
// weight layout.
constexpr int kRowsKC = 256;                       // k per chunk
constexpr int kRowsStride = kRowsKC * 2 + 16;      // bytes per staged activation row

// KSP (layers with few columns): K is also split over a.ksplit workgroups per column group, exchanged as in
// rd_linear_kernel (partial tiles stored write-through, last arriver sums in split order).
template <typename T, int MT, bool TILED, int EPI = EPI_HEAD, bool KSP = false>
__global__ __launch_bounds__(512) void rd_head_rows_kernel(LinArgs<T> a)
{
    typedef typename Elem16<T>::vec8 vec8;
    constexpr int kSteps = kRowsKC / 32;                               // k-steps per chunk
    constexpr int kMine = kSteps / 2;                                  // ... of which a wave takes half
    constexpr int kBuf = MT * 16 * kRowsStride;                        // bytes per buffer
    constexpr int kPieces = MT * 16 * (kRowsKC * 2 / 16) / 512;        // 16-byte pieces per thread and chunk
    extern __shared__ __align__(16) unsigned char s_x[];               // two buffers
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int cp = wave & 3, kh = wave >> 2;                           // column pair, half of every chunk's k-steps
    const int r16 = lane & 15, g = lane >> 4;
    const int groups = KSP ? (int)gridDim.x / a.ksplit : (int)gridDim.x;
    const int group = KSP ? (int)blockIdx.x % groups : (int)blockIdx.x;
    const int split = KSP ? (int)blockIdx.x / groups : 0;
    const int n_tile = (group * 8 + cp * 2) * 16;                      // this wave's 32 columns: tiles n_tile, n_tile + 16
    // this workgroup's chunks of K: [c_first, c_first + nchunks)
    const int all_chunks = a.K1 / kRowsKC;
    const int c_first = KSP ? all_chunks * split / a.ksplit : 0;
    const int nchunks = KSP ? all_chunks * (split + 1) / a.ksplit - c_first : all_chunks;

    const T *wp[2];                                                    // this lane's first weight vector of either tile
    constexpr int wstep = TILED ? 512 : 32;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        if (TILED) {
            const int ntile = min(n_tile / 16 + t, (a.N + 15) / 16 - 1);   // tiles past N read the last one; never stored
            wp[t] = a.w1 + (size_t)ntile * (a.K1 >> 5) * 512 + lane * 8 + (c_first * kSteps + kh * kMine) * wstep;
        } else {
            wp[t] = a.w1 + (size_t)min(n_tile + t * 16 + r16, a.N - 1) * a.K1 + 8 * g + (c_first * kSteps + kh * kMine) * wstep;
        }
    }
    const T *xsrc[kPieces];
    int xdst[kPieces];
#pragma unroll
    for (int i = 0; i < kPieces; ++i) {
        const int p = tid + 512 * i, row = p >> 5, ch = p & 31;
        const size_t prow = (size_t)(a.m0 + min(row, a.M - 1)) * a.mstride;
        xsrc[i] = a.x1 + prow * a.ldx1 + ch * 8 + c_first * kRowsKC;
        xdst[i] = row * kRowsStride + ch * 16;
    }
    f32x4 acc[MT][2];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) acc[mt][0] = acc[mt][1] = f32x4{0.f, 0.f, 0.f, 0.f};

    // (staged values are kept as native vectors: arrays of those stay in registers)
    vec8 wa0[2][kMine], wa1[2][kMine];
    {   // chunk 0: activations -> buffer 0, weights -> wa0
        vec8 x0[kPieces];
#pragma unroll
        for (int i = 0; i < kPieces; ++i) x0[i] = *reinterpret_cast<const vec8 *>(xsrc[i]);
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int s = 0; s < kMine; ++s) wa0[t][s] = *reinterpret_cast<const vec8 *>(wp[t] + s * wstep);
#pragma unroll
        for (int i = 0; i < kPieces; ++i) *reinterpret_cast<vec8 *>(s_x + xdst[i]) = x0[i];
    }

    const int b_off = r16 * kRowsStride + g * 16 + kh * kMine * 64;    // B operand: row r16 of a tile, k group g, own k-steps
    auto chunk = [&](int c, vec8 (&cur)[2][kMine], vec8 (&nxt)[2][kMine]) __attribute__((always_inline)) {
        // the next chunk's activations and weights (after the last chunk: the last chunk again, ignored)
        const int cn = min(c + 1, nchunks - 1);
        vec8 xs[kPieces];
#pragma unroll
        for (int i = 0; i < kPieces; ++i) xs[i] = *reinterpret_cast<const vec8 *>(xsrc[i] + cn * kRowsKC);
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int s = 0; s < kMine; ++s) nxt[t][s] = *reinterpret_cast<const vec8 *>(wp[t] + (cn * kSteps + s) * wstep);
        rd_lds_barrier();                                              // buffer c&1 is complete, buffer (c+1)&1 is free
        const unsigned char *buf = s_x + (c & 1) * kBuf + b_off;
#pragma unroll
        for (int s = 0; s < kMine; ++s) {
            vec8 xb[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) xb[mt] = *reinterpret_cast<const vec8 *>(buf + mt * 16 * kRowsStride + s * 64);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                acc[mt][0] = Elem16<T>::mfma(cur[0][s], xb[mt], acc[mt][0]);
                acc[mt][1] = Elem16<T>::mfma(cur[1][s], xb[mt], acc[mt][1]);
            }
        }
        unsigned char *dst = s_x + ((c + 1) & 1) * kBuf;
#pragma unroll
        for (int i = 0; i < kPieces; ++i) *reinterpret_cast<vec8 *>(dst + xdst[i]) = xs[i];
    };
    for (int c = 0; c < nchunks; c += 2) {
        chunk(c, wa0, wa1);
        if (c + 1 < nchunks) chunk(c + 1, wa1, wa0);
    }
    // the two halves of k meet in LDS (the staging buffers are free after one more barrier)
    rd_lds_barrier();
    f32x4 *s_acc = reinterpret_cast<f32x4 *>(s_x) + (size_t)cp * MT * 2 * 64 + lane;
    if (kh == 1) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            s_acc[(mt * 2 + 0) * 64] = acc[mt][0];
            s_acc[(mt * 2 + 1) * 64] = acc[mt][1];
        }
    }
    rd_lds_barrier();
    if constexpr (!KSP) {
        if (kh == 1) return;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            linear_epilogue<T, EPI>(a, acc[mt][0] + s_acc[(mt * 2 + 0) * 64], mt * 16, n_tile, r16, g);
            linear_epilogue<T, EPI>(a, acc[mt][1] + s_acc[(mt * 2 + 1) * 64], mt * 16, n_tile + 16, r16, g);
        }
    } else {
        // this workgroup's tiles, numbered as an MT x 8 grid (row tile, column tile), -> workspace
        constexpr int kTiles = MT * 8;
        if (kh == 0) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    const f32x4 v = acc[mt][t] + s_acc[(mt * 2 + t) * 64];
                    const int id = mt * 8 + cp * 2 + t;
                    rd::st_dev4(a.kpart + ((((size_t)group * a.ksplit + split) * kTiles + id) * 64 + lane) * 4, v[0], v[1], v[2], v[3]);
                }
        }
        __shared__ uint32_t s_last;
        rd::wait_dev_stores();
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");      // this workgroup's partial tiles are acknowledged
        __syncthreads();
        if (tid == 0) {
            const uint32_t prev = __hip_atomic_fetch_add(a.kcount + group, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            s_last = (prev + 1u == (uint32_t)a.ksplit) ? 1u : 0u;
            if (s_last) a.kcount[group] = 0;                        // ready for the next launch
        }
        __syncthreads();
        if (!s_last) return;
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
        const int n0 = group * 128;
        if (a.ksplit == 8) linear_finish_split<T, MT, 8, 8, EPI, 8>(a, group, n0, wave, lane);
        else if (a.ksplit == 4) linear_finish_split<T, MT, 8, 8, EPI, 4>(a, group, n0, wave, lane);
        else linear_finish_split<T, MT, 8, 8, EPI, 2>(a, group, n0, wave, lane);
    }
}

// rows m = b*W + w: X0 = [e(last token), h] (fp32 and bf16), state = e(last token), path = [last token]
template <typename T>
__global__ void rd_draft_init_kernel(const T *__restrict__ emb, const T *__restrict__ h,
                                     const int32_t *__restrict__ last_token, int W, int L, int Dm, int V,
                                     float *__restrict__ x_f32, T *__restrict__ x_bf, T *__restrict__ s_bf,
                                     int32_t *__restrict__ paths, float *__restrict__ cum, uint32_t *__restrict__ kcount)
{
    const int m = blockIdx.x, b = m / W;
    if (m == 0 && kcount)                                      // arrival counters of the split linear layers
        for (int i = threadIdx.x; i < kSplitMaxGroups; i += blockDim.x) kcount[i] = 0;
    int tok = last_token[b];
    tok = tok < 0 ? 0 : (tok > V - 1 ? V - 1 : tok);
    for (int i = threadIdx.x * 8; i < Dm; i += blockDim.x * 8) {          // Dm is a multiple of 64
        typedef typename Elem16<T>::vec8 vec8;
        const vec8 e = *reinterpret_cast<const vec8 *>(emb + (size_t)tok * Dm + i);
        const vec8 hv = *reinterpret_cast<const vec8 *>(h + (size_t)b * Dm + i);
        *reinterpret_cast<vec8 *>(x_bf + (size_t)m * 2 * Dm + i) = e;
        *reinterpret_cast<vec8 *>(x_bf + (size_t)m * 2 * Dm + Dm + i) = hv;
        *reinterpret_cast<vec8 *>(s_bf + (size_t)m * Dm + i) = e;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            x_f32[(size_t)m * 2 * Dm + i + j] = (float)e[j];
            x_f32[(size_t)m * 2 * Dm + Dm + i + j] = (float)hv[j];
        }
    }
    for (int j = threadIdx.x; j < L; j += blockDim.x) paths[(size_t)m * L + j] = tok;
    if (threadIdx.x == 0) cum[m] = 0.f;
}

__device__ __forceinline__ bool better(float v, int i, float bv, int bi) { return v > bv || (v == bv && i < bi); }

// Selection here is always a merge of sorted lists, one list per lane: every round the lanes offer
// the heads of their lists, the largest value wins and, among equal values, the lowest lane (lists are
// laid out so that a lower lane means a smaller candidate or smaller tokens, which is the tie rule).
// A round is a maximum over lanes by data-parallel primitives, a ballot and a find-first-set; only the
// winning lane fetches a new head.
template <int kCtrl>
__device__ __forceinline__ float max_step_dpp(float x)
{
    return fmaxf(x, __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(x), __float_as_int(x), kCtrl, 0xf, 0xf, false)));
}
// maximum over each group of 8 consecutive lanes
__device__ __forceinline__ float group8_max(float x)
{
    x = max_step_dpp<0xB1>(x);          // quad_perm [1,0,3,2]: partner lane ^ 1
    x = max_step_dpp<0x4E>(x);          // quad_perm [2,3,0,1]: partner lane ^ 2
    return max_step_dpp<0x141>(x);      // row_half_mirror: the other quad of the 8
}
// maximum over the 64 lanes, the same value in every lane
__device__ __forceinline__ float wave_max(float x)
{
    x = max_step_dpp<0x140>(group8_max(x));                 // row_mirror: the other half of the 16
    const float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 0));
    const float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 16));
    const float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 32));
    const float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), 48));
    return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}
// lowest lane of the wave whose `offer` is set, -1 if none (uniform)
__device__ __forceinline__ int first_lane(bool offer)
{
    const unsigned long long m = __ballot(offer);
    return m ? __ffsll((long long)m) - 1 : -1;
}

constexpr int kChunk = 4096;            // logits per workgroup of the first top-W pass
constexpr int kChunkThreads = 256;
constexpr int kChunkPer = kChunk / kChunkThreads;
static_assert(kMaxVocab / kChunk <= 64, "one lane per chunk in the row pass");

// Compare-exchange of a sorting network on (value, position) pairs: the better pair goes to a.
__device__ __forceinline__ void order_pair(float &va, int &ka, float &vb, int &kb)
{
    const bool swap = better(vb, kb, va, ka);
    const float tv = swap ? vb : va, uv = swap ? va : vb;
    const int tk = swap ? kb : ka, uk = swap ? ka : kb;
    va = tv; vb = uv; ka = tk; kb = uk;
}

// First pass over the logits: workgroup (chunk c, row m) reduces 4096 logits to their maximum, the
// sum of exp(x - maximum) and their W best (value, then smaller token).  A lane owns 16 consecutive
// tokens and sorts them in registers (odd-even merge sort network); the sorted lists go to LDS.  Each
// wave merges its 64 lists into its W best, wave 0 then merges the four waves' lists.
__global__ __launch_bounds__(kChunkThreads) void rd_topw_chunk_kernel(const float *__restrict__ logits, int V, int W, int chunks, int mstride, int lpc,
                                                                      float *__restrict__ part_max, float *__restrict__ part_sum,
                                                                      float *__restrict__ part_cv, int32_t *__restrict__ part_ci)
{
    constexpr int kWaves = kChunkThreads / 64;
    __shared__ float s_v[kWaves];
    __shared__ float s_mx;
    __shared__ float s_lv[kChunkPer][kChunkThreads];        // sorted lists, position-major (a lane's column)
    __shared__ unsigned char s_lk[kChunkPer][kChunkThreads];
    __shared__ float s_cv[kWaves][kMaxBeam];
    __shared__ int s_ci[kWaves][kMaxBeam];
    const int c = blockIdx.x, m = blockIdx.y * mstride, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float *z = logits + (size_t)m * V;
    const int t0 = c * kChunk + tid * kChunkPer;            // this lane's first token
    float x[kChunkPer];
    int k[kChunkPer];
    if ((V & 3) == 0 && t0 + kChunkPer <= V) {
#pragma unroll
        for (int j = 0; j < kChunkPer; j += 4) {
            const float4 q = *reinterpret_cast<const float4 *>(z + t0 + j);
            x[j] = q.x; x[j + 1] = q.y; x[j + 2] = q.z; x[j + 3] = q.w;
        }
    } else {
#pragma unroll
        for (int j = 0; j < kChunkPer; ++j) x[j] = t0 + j < V ? z[t0 + j] : -INFINITY;
    }
    int n_valid = V - t0;
    n_valid = n_valid < 0 ? 0 : (n_valid > kChunkPer ? kChunkPer : n_valid);
    float mx = -INFINITY;
#pragma unroll
    for (int j = 0; j < kChunkPer; ++j) { k[j] = j; mx = fmaxf(mx, x[j]); }
    mx = wave_max(mx);
    if (lane == 0) s_v[wave] = mx;
    __syncthreads();
    if (tid == 0) s_mx = fmaxf(fmaxf(s_v[0], s_v[1]), fmaxf(s_v[2], s_v[3]));
    __syncthreads();
    mx = s_mx;
    float sum = 0.f;
#pragma unroll
    for (int j = 0; j < kChunkPer; ++j) sum += j < n_valid ? __expf(x[j] - mx) : 0.f;
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off, 64);
    __syncthreads();
    if (lane == 0) s_v[wave] = sum;

    // sort the lane's 16 (value, position) pairs, best first (Batcher's odd-even merge sort);
    // positions past the end of the vocabulary hold -inf and, being later positions, sort behind
    // real tokens of the same value
#pragma unroll
    for (int pp = 1; pp < kChunkPer; pp <<= 1)
#pragma unroll
        for (int kk = pp; kk >= 1; kk >>= 1)
#pragma unroll
            for (int jj = kk % pp; jj + kk < kChunkPer; jj += 2 * kk)
#pragma unroll
                for (int ii = 0; ii < kk; ++ii)
                    if (ii + jj + kk < kChunkPer && (ii + jj) / (2 * pp) == (ii + jj + kk) / (2 * pp))
                        order_pair(x[ii + jj], k[ii + jj], x[ii + jj + kk], k[ii + jj + kk]);
#pragma unroll
    for (int j = 0; j < kChunkPer; ++j) {
        s_lv[j][tid] = x[j];
        s_lk[j][tid] = (unsigned char)k[j];
    }
    // (a lane reads back only its own column: no barrier needed before the merge)

    // merge of the wave's 64 lists.  Every lane keeps its head and the entry behind it in registers, so
    // a winner moves on without waiting for LDS; the read that refills the second register is only
    // waited for when the same lane wins again.
    float hv = n_valid > 0 ? x[0] : -INFINITY, nv = x[1];
    int hk = k[0], nk = k[1], ptr = 0;
    bool live = n_valid > 0;
    for (int r = 0; r < W; ++r) {
        const float best = wave_max(live ? hv : -INFINITY);
        const int win = first_lane(live && hv == best);
        if (win < 0) {                                      // fewer than W tokens in this wave's range
            if (lane == 0) { s_cv[wave][r] = -INFINITY; s_ci[wave][r] = 0x7fffffff; }
            continue;
        }
        const int wk = __builtin_amdgcn_readlane(hk, win);
        if (lane == 0) {
            s_cv[wave][r] = best;
            s_ci[wave][r] = c * kChunk + (wave * 64 + win) * kChunkPer + wk;
        }
        if (lane == win) {
            ++ptr;
            live = ptr < n_valid;
            hv = nv; hk = nk;
            const int nx = ptr + 1 < kChunkPer ? ptr + 1 : kChunkPer - 1;
            nv = s_lv[nx][tid]; nk = s_lk[nx][tid];
        }
    }
    __syncthreads();
    const size_t slot = (size_t)m * chunks + c;
    if (lpc == kChunkThreads / 64) {
        // wide beams: the four waves' lists leave as they are (the row pass merges four times as many
        // lists in the same number of rounds, and the W rounds of the merge below are saved)
        if (tid == 0) {
            part_max[slot] = mx;
            part_sum[slot] = s_v[0] + s_v[1] + s_v[2] + s_v[3];
        }
        for (int r = lane; r < W; r += 64) {
            part_cv[(slot * lpc + wave) * W + r] = s_cv[wave][r];
            part_ci[(slot * lpc + wave) * W + r] = s_ci[wave][r];
        }
        return;
    }
    if (wave != 0) return;
    if (lane == 0) {
        part_max[slot] = mx;
        part_sum[slot] = s_v[0] + s_v[1] + s_v[2] + s_v[3];
    }
    // merge of the four waves' lists (a lower wave holds smaller tokens): lanes 0..3
    int p4 = 0;
    const int l4 = lane & (kWaves - 1);
    float h4 = s_cv[l4][0], n4 = s_cv[l4][W > 1 ? 1 : 0];
    int i4 = s_ci[l4][0], j4 = s_ci[l4][W > 1 ? 1 : 0];
    bool live4 = lane < kWaves && i4 != 0x7fffffff;
    for (int r = 0; r < W; ++r) {
        const float best = wave_max(live4 ? h4 : -INFINITY);
        const int win = first_lane(live4 && h4 == best);
        if (win < 0) {
            if (lane == 0) { part_cv[slot * W + r] = -INFINITY; part_ci[slot * W + r] = 0x7fffffff; }
            continue;
        }
        if (lane == win) {
            part_cv[slot * W + r] = best;
            part_ci[slot * W + r] = i4;
            ++p4;
            h4 = n4; i4 = j4;
            live4 = p4 < W && i4 != 0x7fffffff;
            const int nx = p4 + 1 < W ? p4 + 1 : W - 1;
            n4 = s_cv[l4][nx]; j4 = s_ci[l4][nx];
        }
    }
}

// Second pass, one lane per (row, chunk): the row's log-sum-exp from the chunk partials and its W best
// tokens as a merge of the chunks' sorted lists (a lower chunk holds smaller tokens), written as
// cumulative scores row_score[row][r] = cum[row] + log p(token r), best first, with the tokens beside
// them.  LPR lanes serve a row: 8 (eight rows per wave) while the vocabulary has at most eight chunks,
// else 64 (one row per wave).
template <int LPR, int WMAX>
__global__ __launch_bounds__(kSelThreads) void rd_topw_row_kernel(
    const float *__restrict__ part_max, const float *__restrict__ part_sum, const float *__restrict__ part_cv,
    const int32_t *__restrict__ part_ci, int chunks, int lpc, const float *__restrict__ cum_cur, int W, int n_rows, int mstride,
    float *__restrict__ row_score, int32_t *__restrict__ row_tok)
{
    constexpr int kRows = 64 / LPR;                                   // rows per wave
    __shared__ float s_cv[64 * WMAX];                                 // [row in wave][chunk][W], LPR * WMAX per row
    __shared__ int s_ci[64 * WMAX];
    const int tid = threadIdx.x, lane = tid & 63, g = lane / LPR, c = lane % LPR;
    const int row_l = blockIdx.x * kRows + g;                         // logical row of this lane's group
    const bool row_ok = row_l < n_rows;
    const size_t row = (size_t)(row_ok ? row_l : n_rows - 1) * mstride;
    const int n_lists = chunks * lpc;                                 // sorted lists per row (lpc per chunk), lane c holds list c
    const int n_surv = n_lists * W;
    auto group_max = [](float x) { return LPR == 8 ? group8_max(x) : wave_max(x); };
    // log-sum-exp of the row: sum_c part_sum[c] * exp(part_max[c] - max) (loads issued before the staging below)
    const bool lane_ok = row_ok && c < chunks;
    const float pm = lane_ok ? part_max[row * chunks + c] : -INFINITY;
    const float gm = group_max(pm);
    float ps = lane_ok ? part_sum[row * chunks + c] * __expf(pm - gm) : 0.f;
#pragma unroll
    for (int off = 1; off < LPR; off <<= 1) ps += __shfl_xor(ps, off, 64);
    const float lse = gm + __logf(ps);
    const float base = row_ok ? cum_cur[row] : 0.f;
    // the survivors of the workgroup's rows -> LDS, by all four waves (one wave alone would spend most of
    // the kernel here at wide beams); eight loads per lane in flight together, addresses past the end
    // pulled back (no load sits behind a branch)
    {
        const int rows_here = min(kRows, n_rows - blockIdx.x * kRows);
        const int total = rows_here * n_surv;
        for (int i0 = 0; i0 < total; i0 += kSelThreads * 8) {
            float v[8];
            int ti[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int idx = min(i0 + u * kSelThreads + tid, total - 1);
                const int gg = idx / n_surv, q = idx - gg * n_surv;
                const size_t src = (size_t)(blockIdx.x * kRows + gg) * mstride * n_surv + q;
                v[u] = part_cv[src];
                ti[u] = part_ci[src];
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int idx = i0 + u * kSelThreads + tid;
                if (idx < total) {
                    const int gg = idx / n_surv, q = idx - gg * n_surv;
                    s_cv[gg * LPR * WMAX + q] = v[u];
                    s_ci[gg * LPR * WMAX + q] = ti[u];
                }
            }
        }
    }
    __syncthreads();
    if (tid >= 64) return;                                            // the merge is one wave's work

    const float *lv = s_cv + g * LPR * WMAX + c * W;                  // this lane's list: chunk c of its row
    const int *li = s_ci + g * LPR * WMAX + c * W;
    int ptr = 0;
    int ht = li[0], nt = li[W > 1 ? 1 : 0];                           // head and the entry behind it, in registers
    float hv = lv[0], nv = lv[W > 1 ? 1 : 0];
    bool live = row_ok && c < n_lists && ht != 0x7fffffff;
    for (int r = 0; r < W; ++r) {
        const float best = group_max(live ? hv : -INFINITY);
        const unsigned long long offers = __ballot(live && hv == best);
        int win;                                                      // chunk that wins in this lane's group
        if (LPR == 8) {
            const unsigned mine = (unsigned)(offers >> (g * 8)) & 0xffu;
            win = mine ? __ffs((int)mine) - 1 : -1;
        } else {
            win = offers ? __ffsll((long long)offers) - 1 : -1;
        }
        if (c == 0 && row_ok) {
            row_score[row * W + r] = win >= 0 ? base + (best - lse) : -INFINITY;
        }
        if (c == win) {
            row_tok[row * W + r] = ht;
            ++ptr;
            hv = nv; ht = nt;
            live = ptr < W && ht != 0x7fffffff;
            const int nx = ptr + 1 < W ? ptr + 1 : W - 1;
            nv = lv[nx]; nt = li[nx];
        } else if (c == 0 && win < 0 && row_ok) {
            row_tok[row * W + r] = 0;
        }
    }
}

// Beam step, one wave per sequence: the best W of the live*W (candidate, token) pairs by cumulative
// score.  Every live row's list is sorted (best first; equal scores by smaller token), so this is a
// merge with lane w holding row w's list: ties go to the smaller candidate, and within a row to the
// list order, i.e. the smaller token.  Then the paths, the scores and the row maps of the next RNN
// update are written.  WIDE (more than 64 candidates): lane w also holds row 64 + w's list, which
// loses ties against every first list, and the lists live in dynamic LDS (2 * live * W words).
template <bool WIDE>
__global__ __launch_bounds__(kSelThreads) void rd_beam_step_kernel(
    const float *__restrict__ row_score, const int32_t *__restrict__ row_tok, int V,
    int W, int L, int t, int live,
    const int32_t *__restrict__ paths_cur, int32_t *__restrict__ paths_next, float *__restrict__ cum_next,
    int32_t *__restrict__ parent_row, int32_t *__restrict__ tok_row,
    int32_t *__restrict__ beams_out, float *__restrict__ logp_out /* both NULL except at the last position */)
{
    constexpr int kCap = WIDE ? kMaxBeam : kNarrowBeam;
    __shared__ float s_score_static[WIDE ? 1 : kNarrowBeam * kNarrowBeam];
    __shared__ int s_ctok_static[WIDE ? 1 : kNarrowBeam * kNarrowBeam];
    extern __shared__ __align__(16) unsigned char s_dyn[];
    __shared__ int s_win[kCap], s_tok[kCap], s_ptr[kCap];
    __shared__ float s_winv[kCap];
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63;
    const int n_cand = live * W;
    float *s_score = WIDE ? reinterpret_cast<float *>(s_dyn) : s_score_static;
    int *s_ctok = WIDE ? reinterpret_cast<int *>(s_dyn) + n_cand : s_ctok_static;
    for (int i0 = 0; i0 < n_cand; i0 += kSelThreads * 8) {        // rows b*W .. b*W+live-1 are contiguous
        float v[8];                                               // eight loads per lane in flight together
        int ti[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int idx = min(i0 + u * kSelThreads + tid, n_cand - 1);
            v[u] = row_score[(size_t)b * W * W + idx];
            ti[u] = row_tok[(size_t)b * W * W + idx];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int idx = i0 + u * kSelThreads + tid;
            if (idx < n_cand) { s_score[idx] = v[u]; s_ctok[idx] = ti[u]; }
        }
    }
    __syncthreads();
    if (tid < 64) {                                               // the merge is one wave's work
    // Every lane keeps the head of its list and the entry behind it in registers, so the winner moves
    // on without waiting for LDS; the rounds only record (candidate, position in its list) and the
    // tokens are looked up afterwards, W at a time.
    int ptr = 0, ptr2 = 0;
    bool on = lane < live, on2 = WIDE && lane + 64 < live;
    const int la = (on ? lane : 0) * W, lb = (on2 ? lane + 64 : 0) * W;
    float hv = s_score[la], nv = s_score[la + (W > 1 ? 1 : 0)];
    float hv2 = s_score[lb], nv2 = s_score[lb + (W > 1 ? 1 : 0)];
    for (int r = 0; r < W; ++r) {
        float offer = on ? hv : -INFINITY;
        if (WIDE) offer = fmaxf(offer, on2 ? hv2 : -INFINITY);
        const float best = wave_max(offer);
        int win = first_lane(on && hv == best);
        bool second = false;                                      // the winner is a second list (candidate 64 + lane)
        if (WIDE && win < 0) {
            win = first_lane(on2 && hv2 == best);
            second = win >= 0;
        }
        if (win < 0) win = first_lane(on);                        // NaN scores: keep indices in range
        if (WIDE && win < 0) {
            win = first_lane(on2);
            second = win >= 0;
        }
        if (win < 0) win = 0;
        if (lane == win) {
            s_win[r] = second ? lane + 64 : lane;
            s_winv[r] = best;
            if (WIDE && second) {
                s_ptr[r] = ptr2 < W ? ptr2 : W - 1;
                if (on2) {
                    ++ptr2;
                    on2 = ptr2 < W;
                    hv2 = nv2;
                    nv2 = s_score[lb + (ptr2 + 1 < W ? ptr2 + 1 : W - 1)];
                }
            } else {
                s_ptr[r] = ptr < W ? ptr : W - 1;
                if (on) {                                         // (not so only when no list had anything left to offer)
                    ++ptr;
                    on = ptr < W;
                    hv = nv;
                    nv = s_score[la + (ptr + 1 < W ? ptr + 1 : W - 1)];
                }
            }
        }
    }
    }
    __syncthreads();
    for (int r = tid; r < W; r += kSelThreads) {
        const int tk = s_ctok[s_win[r] * W + s_ptr[r]];
        s_tok[r] = tk < 0 ? 0 : (tk > V - 1 ? V - 1 : tk);
    }
    __syncthreads();
    // candidate r: parent pw = s_win[r], new token s_tok[r]
    for (int i = tid; i < W * L; i += kSelThreads) {
        const int r = i / L, j = i - r * L;
        const int pw = s_win[r];
        const size_t src = ((size_t)b * W + pw) * L;
        const int v = j < t ? paths_cur[src + j] : (j == t ? s_tok[r] : paths_cur[src]);
        paths_next[((size_t)b * W + r) * L + j] = v;
        if (beams_out) beams_out[((size_t)b * W + r) * L + j] = v;
    }
    for (int w = tid; w < W; w += kSelThreads) {
        cum_next[(size_t)b * W + w] = s_winv[w];
        parent_row[(size_t)b * W + w] = b * W + s_win[w];
        tok_row[(size_t)b * W + w] = s_tok[w];
        if (logp_out) logp_out[(size_t)b * W + w] = s_winv[w];
    }
}

// Row pass and beam step in one launch, for beams of at most 8 candidates over at most 8 chunks (one wave
// holds a whole sequence: lane = candidate row * 8 + chunk): the rows' sorted lists never leave LDS.  Same
// merges, same tie rules and the same arithmetic as the two kernels above; one workgroup per sequence.
__global__ __launch_bounds__(kSelThreads) void rd_row_beam_kernel(
    const float *__restrict__ part_max, const float *__restrict__ part_sum, const float *__restrict__ part_cv,
    const int32_t *__restrict__ part_ci, int chunks, const float *__restrict__ cum_cur, int V, int W, int L, int t, int live,
    const int32_t *__restrict__ paths_cur, int32_t *__restrict__ paths_next, float *__restrict__ cum_next,
    int32_t *__restrict__ parent_row, int32_t *__restrict__ tok_row,
    int32_t *__restrict__ beams_out, float *__restrict__ logp_out /* both NULL except at the last position */)
{
    constexpr int kW = 8;                                             // candidates, chunks and list length at most
    __shared__ float s_cv[kW * kW * kW];                              // [row][chunk][W]: the chunk pass's lists
    __shared__ int s_ci[kW * kW * kW];
    __shared__ float s_score[kW * kW];                                // [row][W]: the rows' lists, cumulative scores
    __shared__ int s_ctok[kW * kW];
    __shared__ int s_win[kW], s_tok[kW], s_ptr[kW];
    __shared__ float s_winv[kW];
    const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, g = lane >> 3, c = lane & 7;
    const bool row_ok = g < live;
    const size_t row = (size_t)b * W + (row_ok ? g : 0);              // rows b*W .. b*W+live-1 (at the first position: b*W)
    const int n_surv = chunks * W;
    const bool lane_ok = row_ok && c < chunks;
    const float pm = lane_ok ? part_max[row * chunks + c] : -INFINITY;
    const float gm = group8_max(pm);
    float ps = lane_ok ? part_sum[row * chunks + c] * __expf(pm - gm) : 0.f;
#pragma unroll
    for (int off = 1; off < 8; off <<= 1) ps += __shfl_xor(ps, off, 64);
    const float lse = gm + __logf(ps);
    const float base = row_ok ? cum_cur[row] : 0.f;
    {   // the sequence's survivors -> LDS (two loads per thread in flight, addresses past the end pulled back)
        const int total = live * n_surv;                              // <= 512
        float v[2];
        int ti[2];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int idx = min(u * kSelThreads + tid, total - 1);
            const int gg = idx / n_surv, q = idx - gg * n_surv;
            const size_t src = ((size_t)b * W + gg) * n_surv + q;
            v[u] = part_cv[src];
            ti[u] = part_ci[src];
        }
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int idx = u * kSelThreads + tid;
            if (idx < total) {
                const int gg = idx / n_surv, q = idx - gg * n_surv;
                s_cv[gg * kW * kW + q] = v[u];
                s_ci[gg * kW * kW + q] = ti[u];
            }
        }
    }
    __syncthreads();
    if (tid < 64) {
        // rows: merge of each row's chunk lists into its W best tokens, as cumulative scores
        const float *lv = s_cv + g * kW * kW + c * W;
        const int *li = s_ci + g * kW * kW + c * W;
        int ptr = 0;
        int ht = li[0], nt = li[W > 1 ? 1 : 0];
        float hv = lv[0], nv = lv[W > 1 ? 1 : 0];
        bool on = lane_ok && ht != 0x7fffffff;
        for (int r = 0; r < W; ++r) {
            const float best = group8_max(on ? hv : -INFINITY);
            const unsigned long long offers = __ballot(on && hv == best);
            const unsigned mine = (unsigned)(offers >> (g * 8)) & 0xffu;
            const int win = mine ? __ffs((int)mine) - 1 : -1;
            if (c == 0 && row_ok) s_score[g * W + r] = win >= 0 ? base + (best - lse) : -INFINITY;
            if (c == win) {
                s_ctok[g * W + r] = ht;
                ++ptr;
                hv = nv; ht = nt;
                on = ptr < W && ht != 0x7fffffff;
                const int nx = ptr + 1 < W ? ptr + 1 : W - 1;
                nv = lv[nx]; nt = li[nx];
            } else if (c == 0 && win < 0 && row_ok) {
                s_ctok[g * W + r] = 0;
            }
        }
    }
    __syncthreads();
    if (tid < 64) {
        // sequence: merge of the live rows' lists, lane w = row w
        int ptr = 0;
        bool on = lane < live;
        const int la = (on ? lane : 0) * W;
        float hv = s_score[la], nv = s_score[la + (W > 1 ? 1 : 0)];
        for (int r = 0; r < W; ++r) {
            const float best = wave_max(on ? hv : -INFINITY);
            int win = first_lane(on && hv == best);
            if (win < 0) win = first_lane(on);                        // NaN scores: keep indices in range
            if (win < 0) win = 0;
            if (lane == win) {
                s_win[r] = lane;
                s_winv[r] = best;
                s_ptr[r] = ptr < W ? ptr : W - 1;
                if (on) {
                    ++ptr;
                    on = ptr < W;
                    hv = nv;
                    nv = s_score[la + (ptr + 1 < W ? ptr + 1 : W - 1)];
                }
            }
        }
    }
    __syncthreads();
    for (int r = tid; r < W; r += kSelThreads) {
        const int tk = s_ctok[s_win[r] * W + s_ptr[r]];
        s_tok[r] = tk < 0 ? 0 : (tk > V - 1 ? V - 1 : tk);
    }
    __syncthreads();
    for (int i = tid; i < W * L; i += kSelThreads) {
        const int r = i / L, j = i - r * L;
        const int pw = s_win[r];
        const size_t src = ((size_t)b * W + pw) * L;
        const int v = j < t ? paths_cur[src + j] : (j == t ? s_tok[r] : paths_cur[src]);
        paths_next[((size_t)b * W + r) * L + j] = v;
        if (beams_out) beams_out[((size_t)b * W + r) * L + j] = v;
    }
    for (int w = tid; w < W; w += kSelThreads) {
        cum_next[(size_t)b * W + w] = s_winv[w];
        parent_row[(size_t)b * W + w] = b * W + s_win[w];
        tok_row[(size_t)b * W + w] = s_tok[w];
        if (logp_out) logp_out[(size_t)b * W + w] = s_winv[w];
    }
}

// For every final candidate, the row of each position's logit matrix that produced its token there:
// follow the parent rows back from the last position.  One thread per candidate.
__global__ void rd_draft_rows_kernel(const int32_t *__restrict__ parents /*[T][M]*/, int M, int W, int T,
                                     int32_t *__restrict__ step_row /*[B][W][T]*/)
{
    const int m = blockIdx.x * blockDim.x + threadIdx.x;
    if (m >= M) return;
    int r = m;
    for (int t = T; t >= 1; --t) {
        r = parents[(size_t)(t - 1) * M + r];
        r = r < 0 ? 0 : (r > M - 1 ? M - 1 : r);
        step_row[(size_t)m * T + t - 1] = r;
    }
}

// Operand-tiled weight layout: the matrix [N][K] (row-major, 16-bit elements) cut into tiles of 16
// rows x 32 columns, tile (n/16, k/32) stored as the 1 KB a wave loads for one MFMA A operand -- lane
// (row n%16, column group g = (k%32)/8) holds its eight consecutive elements at offset lane*8 with
// lane = g*16 + n%16 -- tiles of one row band consecutive in k.  Rows past N are zero.  A wave
// instruction of the linear kernel then reads 1 KB of consecutive memory instead of 64 B from each
// of 16 rows that lie K elements apart.
__global__ void rd_pack_weights_kernel(const uint16_t *__restrict__ src, int N, int K, uint16_t *__restrict__ dst)
{
    const size_t tile = blockIdx.x;                              // (n/16) * (K/32) + k/32
    const int ks = (int)(tile % (size_t)(K >> 5)), nt = (int)(tile / (size_t)(K >> 5));
    const int lane = threadIdx.x, r16 = lane & 15, g = lane >> 4;
    const int n = nt * 16 + r16;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (n < N) v = *reinterpret_cast<const uint4 *>(src + (size_t)n * K + ks * 32 + g * 8);
    *reinterpret_cast<uint4 *>(dst + (tile * 64 + lane) * 8) = v;
}

struct Plan {
    size_t x_f32[3], x_bf[3], s_bf[2], logits, part_max, part_sum, part_cv, part_ci, row_score, row_tok, paths[2], cum[2], parent, tok, kcount, kpart, total;
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
    const size_t chunks = ((size_t)V + kChunk - 1) / kChunk;
    p.part_max = take(M * chunks * 4);
    p.part_sum = take(M * chunks * 4);
    const size_t lists = chunks * 4 <= 64 ? chunks * 4 : chunks;   // wide beams keep four lists per chunk
    p.part_cv = take(M * lists * W * 4);
    p.part_ci = take(M * lists * W * 4);
    p.row_score = take(M * W * 4);
    p.row_tok = take(M * W * 4);
    for (int i = 0; i < 2; ++i) { p.paths[i] = take(M * L * 4); p.cum[i] = take(M * 4); }
    p.parent = take(M * 4 * (size_t)(L > 1 ? L - 1 : 1));       // parent rows of every drafted position
    p.tok = take(M * 4);
    p.kcount = take(kSplitMaxGroups * sizeof(uint32_t));
    p.kpart = take(M > 32 ? (size_t)kSplitMaxWgs * kSplitTiles * 1024 : 0);   // 33 rows and more: layers may split K over workgroups
    p.total = off;
    return p;
}

int draft_check(const rd_draft_params *p, int B, int W, int L)
{
    if (!p || B <= 0 || W <= 0 || L <= 0) return RD_ERR_INVALID_ARG;
    if (p->Dm <= 0 || p->V <= 0 || p->n_mlp < 0) return RD_ERR_INVALID_ARG;
    if (p->Dm % 64 != 0) return RD_ERR_UNSUPPORTED;              // every wave's K share is whole 32-wide steps
    if (p->dtype != RD_BF16 && p->dtype != RD_F16) return RD_ERR_UNSUPPORTED;
    if (p->tiled != 0 && p->tiled != 1) return RD_ERR_INVALID_ARG;
    if (W > kMaxBeam || (long long)B * W > kMaxRows || W > p->V) return RD_ERR_UNSUPPORTED;
    if (p->V > kMaxVocab || L > RD_MAX_N) return RD_ERR_UNSUPPORTED;
    return RD_OK;
}

template <typename T, int MT, int NT, int NWV, int EPI>
void launch_linear_one(const LinArgs<T> &a, hipStream_t stream)
{
    if (a.tiled)
        hipLaunchKernelGGL((rd_linear_kernel<T, MT, NT, NWV, EPI, true>), dim3((a.N + 16 * NT - 1) / (16 * NT)), dim3(NWV * 64), 0, stream, a);
    else
        hipLaunchKernelGGL((rd_linear_kernel<T, MT, NT, NWV, EPI, false>), dim3((a.N + 16 * NT - 1) / (16 * NT)), dim3(NWV * 64), 0, stream, a);
}

// waves per workgroup: as many as give the launch about 16 waves per compute unit, as long as
// every wave gets whole k-steps inside one product and its registers allow that many residents
template <typename T, int MT, int NT, int EPI>
int launch_linear_nt(const LinArgs<T> &a, hipStream_t stream)
{
    const int ks1 = a.K1 / 32, ks2 = a.K2 / 32, wgs = (a.N + 16 * NT - 1) / (16 * NT);
    auto ok = [&](int nwv) {
        if (ks2 == 0) return ks1 % nwv == 0;
        return ks1 == ks2 && ks1 % (nwv / 2) == 0;
    };
    int nwv = 4;
    if (wgs * 4 < 4096 && ok(8)) nwv = 8;
    if (wgs * 8 < 4096 && ok(16)) nwv = 16;
    constexpr bool k16 = MT * NT <= 4 && MT + NT <= 5;          // 16 waves need <= 128 registers per lane
    if (nwv == 16) { if constexpr (k16) launch_linear_one<T, MT, NT, 16, EPI>(a, stream); else launch_linear_one<T, MT, NT, 8, EPI>(a, stream); }
    else if (nwv == 8) launch_linear_one<T, MT, NT, 8, EPI>(a, stream);
    else launch_linear_one<T, MT, NT, 4, EPI>(a, stream);
    return rd_check_launch();
}

// Layers with few columns at 17 rows and more: the widest workgroups the registers allow, and K
// split over as many workgroups per column group as bring the launch to about one workgroup per
// compute unit.  False if the shape does not fit (the caller then takes the unsplit kernels).
template <typename T, int MT, int EPI>
bool launch_linear_split(const LinArgs<T> &a, hipStream_t stream, int *status)
{
    if constexpr (MT >= 4 && EPI != EPI_HEAD) {
        constexpr int NT = MT == 8 ? 4 : 8;
        static_assert(MT * NT <= kSplitTiles, "partial tiles per workgroup");
        constexpr int NWV = 8;                                  // 512 threads: <= 256 registers per lane, no accumulation registers
        static const int ks_env = rd::env_int("RD_DRAFT_KSPLIT", 0);       // 1: never split; 2, 4, 8: only that split
        constexpr int max_wgs = kSplitMaxWgs;                   // one workgroup of 8 waves per compute unit at this register count
        if (a.kpart == nullptr || ks_env == 1) return false;
        if constexpr (EPI == EPI_MLP) {                         // column-split waves, activations through LDS
            static const int rows_on = rd::env_int("RD_DRAFT_MLP_ROWS", 1);
            const int g128 = (a.N + 127) / 128, chunks = a.K1 / kRowsKC;
            int sp = 0;
            for (int c = 8; c >= 2 && sp == 0; c >>= 1)
                if ((ks_env == 0 || ks_env == c) && g128 * c <= kSplitMaxWgs && chunks >= c) sp = c;
            if (rows_on && a.K2 == 0 && a.map1 == nullptr && a.K1 % kRowsKC == 0 && g128 <= kSplitMaxGroups && sp) {
                constexpr size_t smem = 2 * (size_t)MT * 16 * kRowsStride;
                static std::atomic<unsigned long long> conf_t{0}, conf_r{0};
                const void *fn = a.tiled ? reinterpret_cast<const void *>(&rd_head_rows_kernel<T, MT, true, EPI_MLP, true>)
                                         : reinterpret_cast<const void *>(&rd_head_rows_kernel<T, MT, false, EPI_MLP, true>);
                if (rd::ensure_dynamic_lds(fn, smem, a.tiled ? conf_t : conf_r) != RD_OK) { *status = RD_ERR_HIP; return true; }
                LinArgs<T> b = a;
                b.ksplit = sp;
                const dim3 grid(g128 * sp);
                if (a.tiled) hipLaunchKernelGGL((rd_head_rows_kernel<T, MT, true, EPI_MLP, true>), grid, dim3(512), smem, stream, b);
                else hipLaunchKernelGGL((rd_head_rows_kernel<T, MT, false, EPI_MLP, true>), grid, dim3(512), smem, stream, b);
                *status = rd_check_launch();
                return true;
            }
        }
        const int groups = (a.N + 16 * NT - 1) / (16 * NT);
        if (groups > kSplitMaxGroups) return false;
        const int ks1 = a.K1 / 32, ks = ks1 + a.K2 / 32;
        auto ok = [&](int split) {                              // whole k-steps per wave, inside one product
            if (groups * split > max_wgs || ks % (split * NWV) != 0) return false;
            return a.K2 == 0 || ks1 % (ks / (split * NWV)) == 0;
        };
        int split = 0;
        for (int c = 8; c >= 2 && split == 0; c >>= 1)
            if ((ks_env == 0 || ks_env == c) && ok(c)) split = c;
        if (split == 0) return false;
        LinArgs<T> b = a;
        b.ksplit = split;
        const dim3 grid(groups * split);
        if (a.tiled) hipLaunchKernelGGL((rd_linear_kernel<T, MT, NT, NWV, EPI, true, true>), grid, dim3(NWV * 64), 0, stream, b);
        else hipLaunchKernelGGL((rd_linear_kernel<T, MT, NT, NWV, EPI, false, true>), grid, dim3(NWV * 64), 0, stream, b);
        *status = rd_check_launch();
        return true;
    } else {
        return false;
    }
}

// The output layer at 9 rows and more per launch, wide enough to cover half the chip with 128-column
// workgroups: waves split the columns, activations staged in LDS (rd_head_rows_kernel).  Measured per call
// at a hidden size of 4096 and 32000 tokens against the K-split kernels: 16 rows 832 -> 766 us, 32 rows
// 919 -> 835, 64 rows 1007 -> 965, 128 rows 1400 -> 1173; 8 rows 725 -> 730 (not used there).
template <typename T, int MT, int EPI>
bool launch_head_rows(const LinArgs<T> &a, hipStream_t stream, int *status)
{
    if constexpr (MT >= 1 && EPI == EPI_HEAD) {
        static const int on = rd::env_int("RD_DRAFT_HEAD_ROWS", 1);    // 0: the K-split kernel (for comparisons)
        if (!on || a.K2 != 0 || a.map1 != nullptr || a.K1 % kRowsKC != 0 || a.N < 128 * 128) return false;
        if (a.M <= 8) return false;                                    // up to 8 rows the K-split kernel is as fast or faster
        constexpr size_t smem = 2 * (size_t)MT * 16 * kRowsStride;
        static std::atomic<unsigned long long> conf_t{0}, conf_r{0};
        const void *fn = a.tiled ? reinterpret_cast<const void *>(&rd_head_rows_kernel<T, MT, true>)
                                 : reinterpret_cast<const void *>(&rd_head_rows_kernel<T, MT, false>);
        if (rd::ensure_dynamic_lds(fn, smem, a.tiled ? conf_t : conf_r) != RD_OK) { *status = RD_ERR_HIP; return true; }
        const dim3 grid((a.N + 127) / 128);
        if (a.tiled) hipLaunchKernelGGL((rd_head_rows_kernel<T, MT, true>), grid, dim3(512), smem, stream, a);
        else hipLaunchKernelGGL((rd_head_rows_kernel<T, MT, false>), grid, dim3(512), smem, stream, a);
        *status = rd_check_launch();
        return true;
    } else {
        return false;
    }
}

// column tiles per workgroup: the most that still leave about one workgroup per compute unit (the
// activation re-reads are MT : NT of the weight bytes, and measured they cost as much as the
// weights' own stream; halving the workgroups below the number of compute units costs more)
template <typename T, int MT, int EPI>
int launch_linear_mt(const LinArgs<T> &a, hipStream_t stream)
{
    int status = RD_OK;
    if (launch_linear_split<T, MT, EPI>(a, stream, &status)) return status;
    if (launch_head_rows<T, MT, EPI>(a, stream, &status)) return status;
    if constexpr (MT == 2 || MT == 4) {
        if (a.N >= 240 * 128) return launch_linear_nt<T, MT, 8, EPI>(a, stream);
    }
    if constexpr (MT >= 4) {                                    // (at 113 rows and more even half a chip of these beats narrower ones)
        if (a.N >= (MT == 8 ? 128 : 256) * 64) return launch_linear_nt<T, MT, 4, EPI>(a, stream);
    }
    if constexpr (MT >= 2) {
        if (a.N >= 256 * 32) return launch_linear_nt<T, MT, 2, EPI>(a, stream);
    }
    return launch_linear_nt<T, MT, 1, EPI>(a, stream);
}

// more than 128 rows: one launch per 128 rows (each streams the weights again)
template <typename T, int EPI>
int launch_linear(const LinArgs<T> &all, hipStream_t stream)
{
    for (int m0 = 0; m0 < all.M; m0 += kRowsPerLaunch) {
        LinArgs<T> a = all;
        a.m0 = m0;
        a.M = all.M - m0 < kRowsPerLaunch ? all.M - m0 : kRowsPerLaunch;
        const int mt = (a.M + 15) / 16;
        int st;
        if (mt <= 1) st = launch_linear_mt<T, 1, EPI>(a, stream);
        else if (mt <= 2) st = launch_linear_mt<T, 2, EPI>(a, stream);
        else if (mt <= 4) st = launch_linear_mt<T, 4, EPI>(a, stream);
        else st = launch_linear_mt<T, 8, EPI>(a, stream);
        if (st != RD_OK) return st;
    }
    return RD_OK;
}

// The whole call for one storage type (launches only; arguments already checked).
template <typename E>
int draft_run(const rd_draft_params *p, const void *h, const int32_t *last_token, int B, int W, int L,
              int32_t *beams, float *beam_logp, float *step_logits, int32_t *step_row,
              void *workspace, size_t workspace_bytes, void *stream)
{
    const Plan plan = draft_plan(B, W, L, p->Dm, p->V);
    if (!workspace || !rd_aligned(workspace, 256) || workspace_bytes < plan.total) return RD_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    unsigned char *ws = static_cast<unsigned char *>(workspace);
    const int Dm = p->Dm, G = 2 * Dm, V = p->V, M = B * W, T = L - 1;
    float *x_f32[3];
    E *x_bf[3], *s_bf[2];
    for (int i = 0; i < 3; ++i) { x_f32[i] = reinterpret_cast<float *>(ws + plan.x_f32[i]); x_bf[i] = reinterpret_cast<E *>(ws + plan.x_bf[i]); }
    for (int i = 0; i < 2; ++i) s_bf[i] = reinterpret_cast<E *>(ws + plan.s_bf[i]);
    float *logits = reinterpret_cast<float *>(ws + plan.logits);
    float *part_max = reinterpret_cast<float *>(ws + plan.part_max), *part_sum = reinterpret_cast<float *>(ws + plan.part_sum);
    float *part_cv = reinterpret_cast<float *>(ws + plan.part_cv);
    int32_t *part_ci = reinterpret_cast<int32_t *>(ws + plan.part_ci);
    float *row_score = reinterpret_cast<float *>(ws + plan.row_score);
    int32_t *row_tok = reinterpret_cast<int32_t *>(ws + plan.row_tok);
    const int chunks = (V + kChunk - 1) / kChunk;
    int32_t *paths[2] = {reinterpret_cast<int32_t *>(ws + plan.paths[0]), reinterpret_cast<int32_t *>(ws + plan.paths[1])};
    float *cum[2] = {reinterpret_cast<float *>(ws + plan.cum[0]), reinterpret_cast<float *>(ws + plan.cum[1])};
    int32_t *parent = reinterpret_cast<int32_t *>(ws + plan.parent), *tok = reinterpret_cast<int32_t *>(ws + plan.tok);
    uint32_t *kcount = reinterpret_cast<uint32_t *>(ws + plan.kcount);
    float *kpart = M > 32 ? reinterpret_cast<float *>(ws + plan.kpart) : nullptr;
    const E *emb = static_cast<const E *>(p->emb);

    hipLaunchKernelGGL(rd_draft_init_kernel<E>, dim3(M), dim3(256), 0, s, emb, static_cast<const E *>(h), last_token,
                       W, L, Dm, V, x_f32[0], x_bf[0], s_bf[0], paths[0], cum[0], kcount);
    if (rd_check_launch() != RD_OK) return RD_ERR_HIP;
    if (T == 0) {                                   // nothing to draft: the candidates are the LLM's token alone
        hipLaunchKernelGGL(rd_draft_init_kernel<E>, dim3(M), dim3(256), 0, s, emb, static_cast<const E *>(h), last_token,
                           W, L, Dm, V, x_f32[0], x_bf[0], s_bf[0], beams, beam_logp, kcount);
        return rd_check_launch();
    }
    // the h half of X0 must survive the MLP ping-pong: layers write X1 and X2 only
    int si = 0;                                     // state buffer holding s_t of the live candidates
    for (int t = 1; t <= T; ++t) {
        const int cur = (t - 1) & 1, nxt = t & 1;
        if (t > 1) {                                // s_t = f(U s_{t-1}[parent] + W e(token) + b) -> X0[:, :Dm]
            LinArgs<E> a = {};
            a.w1 = static_cast<const E *>(p->rnn_u); a.x1 = s_bf[si]; a.map1 = parent + (size_t)(t - 2) * M; a.ldx1 = Dm; a.K1 = Dm;
            a.w2 = static_cast<const E *>(p->rnn_w); a.x2 = emb; a.map2 = tok; a.ldx2 = Dm; a.K2 = Dm;
            a.bias = p->rnn_b; a.M = M; a.N = Dm; a.mstride = 1; a.tiled = p->tiled;
            a.y_f32 = x_f32[0]; a.y_bf = x_bf[0]; a.s_bf = s_bf[si ^ 1]; a.ldy = G; a.kpart = kpart; a.kcount = kcount;
            if (launch_linear<E, EPI_RNN>(a, s) != RD_OK) return RD_ERR_HIP;
            si ^= 1;
        }
        // at the first position the W rows of a sequence are one and the same state: compute row b*W only
        const int rows = t == 1 ? B : M, mstride = t == 1 ? W : 1;
        int in = 0;
        for (int k = 0; k < p->n_mlp; ++k) {        // x <- x + f(A_k x + c_k)
            const int out = in == 1 ? 2 : 1;
            LinArgs<E> a = {};
            a.w1 = static_cast<const E *>(p->mlp_w) + (size_t)k * G * G; a.x1 = x_bf[in]; a.ldx1 = G; a.K1 = G;
            a.bias = p->mlp_b + (size_t)k * G; a.M = rows; a.N = G; a.mstride = mstride; a.tiled = p->tiled;
            a.y_f32 = x_f32[out]; a.y_bf = x_bf[out]; a.res = x_f32[in]; a.ldy = G; a.kpart = kpart; a.kcount = kcount;
            if (launch_linear<E, EPI_MLP>(a, s) != RD_OK) return RD_ERR_HIP;
            in = out;
        }
        {                                           // logits
            LinArgs<E> a = {};
            a.w1 = static_cast<const E *>(p->head_w); a.x1 = x_bf[in]; a.ldx1 = G; a.K1 = G;
            if (step_logits) logits = step_logits + (size_t)(t - 1) * M * V;   // every position keeps its matrix
            a.M = rows; a.N = V; a.mstride = mstride; a.tiled = p->tiled; a.y_f32 = logits; a.ldy = V;
            if (launch_linear<E, EPI_HEAD>(a, s) != RD_OK) return RD_ERR_HIP;
        }
        // from 16 candidates on (and while four lists per chunk fit the row pass's 64 lanes) the chunk pass
        // leaves its four waves' lists unmerged
        const int lpc = (W >= 16 && chunks * 4 <= 64) ? 4 : 1;
        hipLaunchKernelGGL(rd_topw_chunk_kernel, dim3(chunks, rows), dim3(kChunkThreads), 0, s, logits, V, W, chunks, mstride, lpc,
                           part_max, part_sum, part_cv, part_ci);
        if (rd_check_launch() != RD_OK) return RD_ERR_HIP;
        const bool last = t == T;
        const bool wide = W > kNarrowBeam;
        const int live = t == 1 ? 1 : W;
        static const int fuse_on = rd::env_int("RD_DRAFT_FUSE_ROW_BEAM", 1);   // 0: the two kernels (for comparisons)
        if (fuse_on && W <= 8 && chunks <= 8 && lpc == 1) {
            hipLaunchKernelGGL(rd_row_beam_kernel, dim3(B), dim3(kSelThreads), 0, s, part_max, part_sum, part_cv, part_ci, chunks,
                               cum[cur], V, W, L, t, live, paths[cur], paths[nxt], cum[nxt], parent + (size_t)(t - 1) * M, tok,
                               last ? beams : nullptr, last ? beam_logp : nullptr);
            if (rd_check_launch() != RD_OK) return RD_ERR_HIP;
            continue;
        }
#define RD_ROW_LAUNCH(LPR, WMAX, grid)                                                                                   \
        hipLaunchKernelGGL((rd_topw_row_kernel<LPR, WMAX>), dim3(grid), dim3(kSelThreads), 0, s, part_max, part_sum, part_cv, part_ci, \
                           chunks, lpc, cum[cur], W, rows, mstride, row_score, row_tok)
        if (chunks * lpc <= 8) {
            if (wide) RD_ROW_LAUNCH(8, kMaxBeam, (rows + 7) / 8); else RD_ROW_LAUNCH(8, kNarrowBeam, (rows + 7) / 8);
        } else {
            if (wide) RD_ROW_LAUNCH(64, kMaxBeam, rows); else RD_ROW_LAUNCH(64, kNarrowBeam, rows);
        }
#undef RD_ROW_LAUNCH
        if (rd_check_launch() != RD_OK) return RD_ERR_HIP;
        if (wide) {
            static std::atomic<unsigned long long> configured{0};
            if (rd::ensure_dynamic_lds(reinterpret_cast<const void *>(&rd_beam_step_kernel<true>), (size_t)kMaxBeam * kMaxBeam * 8,
                                       configured) != RD_OK)
                return RD_ERR_HIP;
            hipLaunchKernelGGL(rd_beam_step_kernel<true>, dim3(B), dim3(kSelThreads), (size_t)live * W * 8, s, row_score, row_tok, V, W, L, t,
                               live, paths[cur], paths[nxt], cum[nxt], parent + (size_t)(t - 1) * M, tok,
                               last ? beams : nullptr, last ? beam_logp : nullptr);
        } else {
            hipLaunchKernelGGL(rd_beam_step_kernel<false>, dim3(B), dim3(kSelThreads), 0, s, row_score, row_tok, V, W, L, t,
                               live, paths[cur], paths[nxt], cum[nxt], parent + (size_t)(t - 1) * M, tok,
                               last ? beams : nullptr, last ? beam_logp : nullptr);
        }
        if (rd_check_launch() != RD_OK) return RD_ERR_HIP;
    }
    if (step_row) {
        hipLaunchKernelGGL(rd_draft_rows_kernel, dim3((M + 255) / 256), dim3(256), 0, s, parent, M, W, T, step_row);
        if (rd_check_launch() != RD_OK) return RD_ERR_HIP;
    }
    return RD_OK;
}

}  // namespace

extern "C" size_t rd_draft_workspace(int B, int W, int L, int Dm, int V)
{
    rd_draft_params p = {};
    p.Dm = Dm; p.V = V; p.dtype = RD_BF16;
    if (draft_check(&p, B, W, L) != RD_OK) return 0;
    return draft_plan(B, W, L, Dm, V).total;
}

extern "C" int rd_draft(const rd_draft_params *p, const void *h, const int32_t *last_token,
                        int B, int W, int L, int32_t *beams, float *beam_logp,
                        float *step_logits, int32_t *step_row,
                        void *workspace, size_t workspace_bytes, void *stream)
{
    const int st = draft_check(p, B, W, L);
    if (st != RD_OK) return st;
    if (!p->emb || !p->rnn_u || !p->rnn_w || !p->rnn_b || !p->head_w || (p->n_mlp > 0 && (!p->mlp_w || !p->mlp_b)))
        return RD_ERR_INVALID_ARG;
    if (!h || !last_token || !beams || !beam_logp) return RD_ERR_INVALID_ARG;
    if ((step_logits == nullptr) != (step_row == nullptr) || !rd_aligned(step_logits, 16)) return RD_ERR_INVALID_ARG;
    if (!rd_aligned(p->emb, 16) || !rd_aligned(p->rnn_u, 16) || !rd_aligned(p->rnn_w, 16) || !rd_aligned(p->mlp_w, 16) ||
        !rd_aligned(p->head_w, 16) || !rd_aligned(h, 16))
        return RD_ERR_INVALID_ARG;
    if (p->dtype == RD_F16)
        return draft_run<_Float16>(p, h, last_token, B, W, L, beams, beam_logp, step_logits, step_row, workspace, workspace_bytes, stream);
    return draft_run<__bf16>(p, h, last_token, B, W, L, beams, beam_logp, step_logits, step_row, workspace, workspace_bytes, stream);
}

extern "C" size_t rd_draft_packed_elems(int N, int K)
{
    if (N <= 0 || K <= 0 || K % 32 != 0) return 0;
    return (size_t)((N + 15) / 16 * 16) * (size_t)K;
}

extern "C" int rd_draft_pack_weights(const void *src, int N, int K, void *dst, void *stream)
{
    if (!src || !dst || N <= 0 || K <= 0) return RD_ERR_INVALID_ARG;
    if (K % 32 != 0) return RD_ERR_UNSUPPORTED;
    if (!rd_aligned(src, 16) || !rd_aligned(dst, 16)) return RD_ERR_INVALID_ARG;
    const size_t tiles = (size_t)((N + 15) / 16) * (size_t)(K / 32);
    if (tiles > 0x7fffffffull) return RD_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(rd_pack_weights_kernel, dim3((unsigned)tiles), dim3(64), 0, (hipStream_t)stream,
                       static_cast<const uint16_t *>(src), N, K, static_cast<uint16_t *>(dst));
    return rd_check_launch();
}
