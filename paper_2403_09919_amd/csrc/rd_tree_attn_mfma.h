// Tree-masked attention on the gfx950 matrix cores for 16-bit K/V (bf16 or fp16): the kernel
// template and its dispatch, instantiated once per element type (rd_tree_attn_bf16.hip,
// rd_tree_attn_f16.hip).  The design is described at the top of rd_tree_attn_bf16.hip.
#pragma once
#include "rd_attn_common.h"
#include <type_traits>

#ifdef RD_TRACE
extern __device__ unsigned long long *rd_trace_buf;     // defined by the including file (RD_TRACE_DEFINE)
#endif

namespace rd {

typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef f32x4 f32x4_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
// 16-bit element types of the MFMA kernels: eight-element operand vector and the matrix instruction
template <typename T> struct Elem;
template <> struct Elem<__bf16> {
    typedef bf16x8 vec8;
    static __device__ __forceinline__ f32x4_t mfma(vec8 a, vec8 b, f32x4_t c) { return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0); }
};
template <> struct Elem<_Float16> {
    typedef f16x8 vec8;
    static __device__ __forceinline__ f32x4_t mfma(vec8 a, vec8 b, f32x4_t c) { return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0); }
};
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

template <int D>
struct Geo {
    static constexpr int kChunks = D / 8;                  // 16-byte chunks per row
    static constexpr int kRowBytes = D * 2;
    static constexpr int kTileKeys = 32;                   // keys per wave per block
    static constexpr int kRowsPerLoad = 64 / kChunks;      // rows one wave-wide 16-byte load covers
    static constexpr int kLoads = kTileKeys / kRowsPerLoad;  // loads per wave per tile
    static constexpr int kTileBytes = kTileKeys * kRowBytes;
    static constexpr int kKSteps = D / 32;                 // MFMA k-steps of the QK^T contraction
    static constexpr int kDTiles = D / 16;
    static constexpr int kDTilesPerWave = kDTiles / 4;
};

// LDS placement of 16-byte chunk c of row `row`: K and Q tiles are read by 16 lanes holding 16
// different rows and one chunk index, V tiles by transpose reads that touch 8 rows x 2 adjacent
// chunks per half-wave; each gets the XOR pattern that spreads its readers over all banks.
template <int D> __device__ __forceinline__ int kswz(int row, int c) { return c ^ (row & (Geo<D>::kChunks - 1)); }
template <int D> __device__ __forceinline__ int vswz(int row, int c)
{
    return ((((c >> 1) ^ (row & (Geo<D>::kChunks / 2 - 1))) << 1) | (c & 1));
}

__device__ __forceinline__ uint4 ldg16(const void *p) { return *reinterpret_cast<const uint4 *>(p); }

// Synchronisation that orders LDS traffic only.  __syncthreads() also waits for every global
// load in flight, which would drain the K/V prefetch at each of the three barriers per block.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}
// Orders this wave's own LDS writes before its own later LDS reads (tiles private to a wave).
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// NW = waves per workgroup (4 or 8).  A block is 32*NW keys; eight waves halve the number of
// sequential blocks of a range, which is what counts when a range is only one or two blocks long.
// max / sum over the four lanes l, l^16, l^32, l^48 (the four 8-key groups of a score tile
// column) with the gfx950 lane-swap instructions: each gives a lane the pair {x[l], x[l^k]}.
__device__ __forceinline__ float quad_max(float x)
{
    auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
    auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float quad_sum(float x)
{
    auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = __uint_as_float(a[0]) + __uint_as_float(a[1]);
    auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

// Rotary embedding of eight elements ("rotate half": element i pairs with element i + D/2), in the
// arithmetic of rd_rope: fp32, every product rounded before the sum, one rounding to the storage
// type.  `x` is this lane's 16-byte chunk, `partner` the chunk D/2 elements away in the same row,
// cs / sn the cosines and sines of the eight pairs; `low`: x is the lower half of the pairs.
template <typename T>
__device__ __forceinline__ uint4 rope8(uint4 x, uint4 partner, const float (&cs)[8], const float (&sn)[8], bool low)
{
    typedef typename Elem<T>::vec8 vec8;
    const vec8 xv = __builtin_bit_cast(vec8, x), pv = __builtin_bit_cast(vec8, partner);
    vec8 y;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const float a = (float)xv[i], b = (float)pv[i];
        const float xc = __fmul_rn(a, cs[i]), ps = __fmul_rn(b, sn[i]);
        float r = low ? __fsub_rn(xc, ps) : __fadd_rn(xc, ps);
        asm volatile("" : "+v"(r));               // an fp32 sum, then one rounding (as rd_rope does)
        y[i] = (T)r;
    }
    return __builtin_bit_cast(uint4, y);
}

// TB = packed-key blocks the launch can need: ceil(N / block keys).  1 for all but the widest beams;
// the mask words of every such block are fetched up front, so the common case should not pay for three.
// PAGED: the context keys and values live in fixed-size pages found through a block table
// (a.block_table, a.page_size, a.max_pages) instead of one dense [B,H,Cmax,D] tensor.
// ROPE: q and k_new arrive unrotated; the kernel applies the rotary embedding at a.position_ids
// to the query rows as it brings them into LDS and to the packed-key tiles as it walks them.
template <typename T, int D, int NQ, int NW, int TB, bool PAGED, bool ROPE = false>
__global__ __launch_bounds__(NW * 64, 2) void rd_tree_attn_mfma_kernel(AttnArgs a)
{
    using G = Geo<D>;
    using vec8 = typename Elem<T>::vec8;
    constexpr int kThreads = NW * 64;
    constexpr int kBlock = NW * G::kTileKeys;                   // keys per block
    constexpr int kRows = NQ * 16;
    constexpr int kDTW = G::kDTiles / NW;                       // d-tiles of the output owned by a wave
    static_assert(kDTW >= 1, "more waves than output d-tiles");
    constexpr int kPF = kRows * (2 + D);                        // floats per partial
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char *sQ = smem;                                   // [kRows][kRowBytes]
    unsigned char *sKV = sQ + kRows * G::kRowBytes;             // NW tiles [32][kRowBytes]
    unsigned char *sP = sKV + NW * G::kTileBytes;               // [NW kt][NQ][64 lanes] x 16 B
    float *sM = reinterpret_cast<float *>(sP + NW * NQ * 64 * 16);  // [NW waves][kRows]
    uint32_t *sVis = reinterpret_cast<uint32_t *>(sM + NW * kRows);   // [NW waves][NQ][64 lanes]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // wave-uniform, kept in a scalar register
    const int r16 = lane & 15;
    const int g = lane >> 4;
    RD_TR(0);

    // ---- which (sequence, head, key range) -------------------------------------------------------
    // Workgroups are dealt round-robin to the 8 XCDs; when the head count allows, all ranges of a
    // head go to one XCD so that Q and the partial results stay in that XCD's L2.  Within an XCD
    // the long context ranges come first and the short packed-key ranges last, so that the
    // compute units are filled with long-running workgroups from the start.
    // The packed keys are either a range of their own (split == S, one more workgroup per head) or,
    // when the context ranges are long (a.fuse_tree), one more block at the end of the last context
    // range; with a single context range the head then has one workgroup and needs no merge.
    const int n_part = a.S + (a.fuse_tree ? 0 : 1);
    // Work items are (head, key range, row group); the row groups of one key range are neighbours
    // in launch order so that they stream the same K/V at the same time (one reads HBM, the others L2).
    const int n_rg = a.n_rg;
    int bh, split, rg;
    {
        const int xcd = a.xcd_remap ? (int)(blockIdx.x & 7) : 0;
        const int k = a.xcd_remap ? (int)(blockIdx.x >> 3) : (int)blockIdx.x;
        const int heads_here = a.xcd_remap ? (a.B * a.H) >> 3 : a.B * a.H;    // heads served by this XCD
        const int per_head = a.S * n_rg;
        const int n_ctx = heads_here * per_head;
        int hl;
        if (k < n_ctx) {
            hl = k / per_head;
            const int r = k - hl * per_head;
            split = r / n_rg;
            rg = r - split * n_rg;
        } else {
            const int r = k - n_ctx;
            hl = r / n_rg;
            rg = r - hl * n_rg;
            split = a.S;
        }
        bh = a.xcd_remap ? hl * 8 + xcd : hl;
    }
    const int b = bh / a.H;
    const int C = clampi(a.ctx_len[b], 0, a.Cmax);
    const int P_all = clampi(a.n_packed[b], 0, a.N);
    // This workgroup's rows are row0 .. row0 + kRows - 1 of the packed rows; P of them are real.
    // A packed row p sees no packed key beyond itself (the mask is lower triangular), so the group
    // needs the packed keys [0, tree_end) only.
    const int row0 = rg * kRows;
    const int P = clampi(P_all - row0, 0, kRows);
    const int Ng = min(kRows, a.N - row0);                 // rows of `out` this group owns
    const int tree_end = min(P_all, row0 + kRows);

    // Blocks this workgroup walks: nA blocks of context keys [k_begin, k_end), then nB blocks of
    // packed keys [0, tree_end).  All of this is wave-uniform.  A group without real rows walks nothing.
    int k_begin = 0, k_end = 0;
    if (split < a.S && P > 0) ctx_range(C, a.S, split, kBlock, &k_begin, &k_end);
    const bool has_tree = (split == a.S) || (a.fuse_tree && split == a.S - 1);
    const int nA = (k_end - k_begin + kBlock - 1) / kBlock;
    const int nB = (has_tree && P > 0) ? (tree_end + kBlock - 1) / kBlock : 0;
    const int nb = nA + nB;
    const unsigned char *Qb = static_cast<const unsigned char *>(a.q) + ((size_t)bh * a.N + row0) * G::kRowBytes;
    // dense cache: this head's rows; paged cache: the page pool (the head is picked inside a page)
    const unsigned char *Kc = static_cast<const unsigned char *>(a.k_cache) + (PAGED ? 0 : (size_t)bh * a.Cmax * G::kRowBytes);
    const unsigned char *Vc = static_cast<const unsigned char *>(a.v_cache) + (PAGED ? 0 : (size_t)bh * a.Cmax * G::kRowBytes);
    const unsigned char *Kn = static_cast<const unsigned char *>(a.k_new) + (size_t)bh * a.N * G::kRowBytes;
    const unsigned char *Vn = static_cast<const unsigned char *>(a.v_new) + (size_t)bh * a.N * G::kRowBytes;
    // ---- all first loads, without branches so that the waits on them stay exact --------------------
    // Order: Q and the tree-mask words (they gate the first score tile), then K, then V.
    constexpr int kQRowsPerPass = kThreads / G::kChunks;
    constexpr int kQPasses = (kRows + kQRowsPerPass - 1) / kQRowsPerPass;
    uint4 qreg[kQPasses];
#pragma unroll
    for (int i = 0; i < kQPasses; ++i) {
        const int row = min(i * kQRowsPerPass + tid / G::kChunks, P - 1);    // rows >= P are zeroed below
        qreg[i] = ldg16(Qb + max(row, 0) * G::kRowBytes + (tid % G::kChunks) * 16);
    }
    // rotary embedding of the query rows: the partner chunk, and the cosines / sines of the row's position
    constexpr int kHalfChunks = G::kChunks / 2;
    uint4 qpart[ROPE ? kQPasses : 1];
    float qcs[ROPE ? kQPasses : 1][8], qsn[ROPE ? kQPasses : 1][8];
    if constexpr (ROPE) {
#pragma unroll
        for (int i = 0; i < kQPasses; ++i) {
            const int row = max(min(i * kQRowsPerPass + tid / G::kChunks, P - 1), 0);
            const int chunk = tid % G::kChunks;
            qpart[i] = ldg16(Qb + row * G::kRowBytes + (chunk ^ kHalfChunks) * 16);
            const int pos = clampi(a.position_ids[(size_t)b * a.N + row0 + row], 0, a.max_pos - 1);
            const float *ct = a.cos_tab + (size_t)pos * (D / 2) + (chunk & (kHalfChunks - 1)) * 8;
            const float *st = a.sin_tab + (size_t)pos * (D / 2) + (chunk & (kHalfChunks - 1)) * 8;
#pragma unroll
            for (int e = 0; e < 8; ++e) { qcs[i][e] = ct[e]; qsn[i][e] = st[e]; }
        }
    }
    // Visibility of this wave's 32 keys, in each packed-key block, for the packed rows this lane
    // scores (row row0 + 16*qt + r16).  Context keys are visible to every row; packed keys per the
    // tree mask: in packed-key block t wave w holds keys 32*(t*NW + w) .. +31, i.e. one half of mask
    // word (t*NW + w)/2.  (Loaded by every workgroup; those without a packed-key block ignore it.)
    constexpr int kTreeBlocks = TB;
    static_assert(TB * kBlock < RD_MAX_N + kBlock, "more packed-key blocks than the largest N has");
    uint64_t mword[kTreeBlocks][NQ];
#pragma unroll
    for (int t = 0; t < kTreeBlocks; ++t) {
        const int word = min((t * NW + wave) >> 1, a.words - 1);
#pragma unroll
        for (int qt = 0; qt < NQ; ++qt)
            mword[t][qt] = a.mask_bits[((size_t)b * a.N + min(row0 + qt * 16 + r16, a.N - 1)) * a.words + word];
    }

    // This wave's slice of a block: coalesced 16-byte loads into registers; a wave-wide load
    // covers 1 KB of consecutive rows.  Rows past the end of the range are redirected to the last
    // valid row (their scores are masked and their probabilities are zero), so the loads carry no
    // predicate.
    uint4 kreg[G::kLoads], vreg[G::kLoads];
    const int ld_row = lane / G::kChunks;
    const int ld_chunk = lane % G::kChunks;
    auto load_tile = [&](const unsigned char *base, int key0, int end, uint4 (&reg)[G::kLoads]) __attribute__((always_inline)) {
        const uint32_t off0 = (uint32_t)(key0 + wave * G::kTileKeys + ld_row) * G::kRowBytes + ld_chunk * 16;
        const uint32_t last_off = (uint32_t)(end - 1) * G::kRowBytes + ld_chunk * 16;
#pragma unroll
        for (int s = 0; s < G::kLoads; ++s) reg[s] = ldg16(base + min(off0 + s * 1024u, last_off));
    };
    // Paged cache: a tile (32 keys, never straddling a page because page_size % 32 == 0) is
    // addressed through the page of its first key.  Tiles beyond the end of the range are
    // redirected to the last tile that holds a key, rows beyond the end to the tile's last valid
    // row.  The page id of the tile to prefetch is itself fetched one iteration earlier, so the
    // scalar load's latency is off the critical path.
    const int head = bh - b * a.H;
    auto ctx_tile_first = [&](int key0, int end) __attribute__((always_inline)) {   // first key of this wave's (redirected) tile
        return min(key0 + wave * G::kTileKeys, ((end - 1) >> 5) << 5);
    };
    auto page_of = [&](int t0) __attribute__((always_inline)) {                 // wave-uniform scalar load
        const int pg = min(t0 / a.page_size, a.max_pages - 1);
        return clampi(a.block_table[(size_t)b * a.max_pages + pg], 0, a.n_pages - 1);
    };
    auto load_tile_paged = [&](const unsigned char *pages, int pid, int t0, int end, uint4 (&reg)[G::kLoads]) __attribute__((always_inline)) {
        const unsigned char *base = pages + (((size_t)pid * a.H + head) * a.page_size + (t0 % a.page_size)) * G::kRowBytes;
        const uint32_t off0 = (uint32_t)ld_row * G::kRowBytes + ld_chunk * 16;
        const uint32_t last_off = (uint32_t)(min(G::kTileKeys, end - t0) - 1) * G::kRowBytes + ld_chunk * 16;
#pragma unroll
        for (int s = 0; s < G::kLoads; ++s) reg[s] = ldg16(base + min(off0 + s * 1024u, last_off));
    };
    int pid_next = 0;         // page of this wave's tile in the block after the current one (paged context only)
    {   // first block; a workgroup with no block at all reads (and ignores) the first row of Q
        const bool ctx = nA > 0;
        if (PAGED && ctx) {
            const int t0 = ctx_tile_first(k_begin, k_end);
            const int pid = page_of(t0);
            load_tile_paged(Kc, pid, t0, k_end, kreg);
            load_tile_paged(Vc, pid, t0, k_end, vreg);
            if (nA > 1) pid_next = page_of(ctx_tile_first(k_begin + kBlock, k_end));
        } else {
            const unsigned char *kb = nb == 0 ? Qb : (ctx ? Kc : Kn);
            const unsigned char *vb = nb == 0 ? Qb : (ctx ? Vc : Vn);
            const int key0 = ctx ? k_begin : 0;
            const int end = nb == 0 ? 1 : (ctx ? k_end : tree_end);
            load_tile(kb, key0, end, kreg);
            load_tile(vb, key0, end, vreg);
        }
    }

    // Visibility of this wave's packed keys (used in the packed-key blocks only).  Of a tile's 32
    // keys this lane scores only the eight with index 4g+i and 16+4g+i, so one byte per block is
    // all it keeps: bit 4*mt+i of byte t (row tile qt) = key 16*mt+4g+i of packed-key block t is
    // visible to row 16*qt+r16.
    // With up to three row tiles the bytes stay in registers.  The larger variants are short of
    // registers: there the bytes are parked in LDS (each lane reads back only what it wrote),
    // because a register that is first used inside the block loop but refilled from scratch memory
    // makes the compiler wait for it, and with it for the K/V tiles in flight, in every iteration.
    constexpr bool kVisInLds = NQ > 3;
    uint32_t vis[NQ];
    static_assert(kTreeBlocks <= 4, "one byte per packed-key block");
#pragma unroll
    for (int qt = 0; qt < NQ; ++qt) {
        uint32_t packed = 0;
        if (qt * 16 + r16 < P) {
#pragma unroll
            for (int t = 0; t < kTreeBlocks; ++t) {
                if (((t * NW + wave) >> 1) < a.words) {
                    const uint32_t v32 = (uint32_t)(mword[t][qt] >> ((wave & 1) * 32));
                    packed |= (((v32 >> (4 * g)) & 0xfu) | (((v32 >> (16 + 4 * g)) & 0xfu) << 4)) << (8 * t);
                }
            }
        }
        if (kVisInLds) {
            sVis[(wave * NQ + qt) * 64 + lane] = packed;
            vis[qt] = 0;
        } else {
            asm volatile("" : "+v"(packed));          // computed here, not sunk into the loop's masked path
            vis[qt] = packed;
        }
    }

#pragma unroll
    for (int i = 0; i < kQPasses; ++i) {
        const int row = i * kQRowsPerPass + tid / G::kChunks;
        if (row < kRows)
            *reinterpret_cast<uint4 *>(sQ + row * G::kRowBytes + kswz<D>(row, tid % G::kChunks) * 16) =
                (row < P) ? (ROPE ? rope8<T>(qreg[i], qpart[i], qcs[i], qsn[i], (tid % G::kChunks) < kHalfChunks) : qreg[i])
                          : make_uint4(0, 0, 0, 0);
    }

    float m_run[NQ], l_run[NQ];
    f32x4 oacc[kDTW][NQ];
#pragma unroll
    for (int qt = 0; qt < NQ; ++qt) {
        m_run[qt] = -INFINITY;
        l_run[qt] = 0.f;
#pragma unroll
        for (int j = 0; j < kDTW; ++j) oacc[j][qt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    unsigned char *my_tile = sKV + wave * G::kTileBytes;
    // Lane-constant LDS offsets.  The XOR swizzles make the offset of load s / k-step t / d-tile dt
    // the XOR of one lane-dependent value with a compile-time constant, so one register serves each
    // family instead of one per member.
    const int k_base = ld_row * G::kRowBytes + kswz<D>(ld_row, ld_chunk) * 16;
    const int v_base = ld_row * G::kRowBytes + vswz<D>(ld_row, ld_chunk) * 16;
    auto k_wr = [&](int s) __attribute__((always_inline)) {    // row s*kRowsPerLoad + ld_row, K swizzle
        return s * 1024 + (k_base ^ (((s * G::kRowsPerLoad) & (G::kChunks - 1)) * 16));
    };
    auto v_wr = [&](int s) __attribute__((always_inline)) {    // same row, V swizzle
        return s * 1024 + (v_base ^ (((s * G::kRowsPerLoad) & (G::kChunks / 2 - 1)) * 32));
    };
    const int kq_base = r16 * G::kRowBytes + kswz<D>(r16, g) * 16;
    auto kq_rd = [&](int t) __attribute__((always_inline)) {   // row r16, chunk 4t+g (rows 16+r16, 16qt+r16 add constants)
        return kq_base ^ (((4 * t) & (G::kChunks - 1)) * 16);
    };
    const int vt_row = 4 * g + (r16 >> 2);
    const int vt_base = vt_row * G::kRowBytes + vswz<D>(vt_row, (r16 & 3) >> 1) * 16 + (r16 & 1) * 8;
    auto vt_rd = [&](int dt) __attribute__((always_inline)) {  // transpose-read address of rows 4g+(r16>>2), d-tile dt
        return vt_base ^ ((dt & (G::kChunks / 2 - 1)) * 32);
    };

    lds_barrier();        // Q visible to all waves
    RD_TR(1);

    const int nqt = (P + 15) >> 4;            // row tiles that hold packed rows; the others are skipped
    const float c_abs = fabsf(a.scale_log2e);
    const bool c_neg = a.scale_log2e < 0.f;

    // The block loop is instantiated twice: for all row tiles, and for the lower half when the
    // packed rows fit there (a padded tile costs as much as a real one, and branches around it
    // would stop the compiler from overlapping LDS reads with the matrix instructions); the
    // five-tile kernel, whose full loop is short of registers, has a third for four tiles.
    auto block_loop = [&](auto nqa_tag) __attribute__((always_inline)) {
        constexpr int NQA = decltype(nqa_tag)::value;
        for (int ib = 0; ib < nb; ++ib) {
            // this block and the one to prefetch: tensors, first key, end of the key range.  After
            // the last block the prefetch repeats it (issued and ignored).
            const bool cur_tree = ib >= nA;
            const int cur_key0 = cur_tree ? (ib - nA) * kBlock : k_begin + ib * kBlock;
            const int cur_end = cur_tree ? tree_end : k_end;
            const int inext = ib + 1 < nb ? ib + 1 : ib;
            const bool next_tree = inext >= nA;
            const unsigned char *next_kb = next_tree ? Kn : Kc;
            const unsigned char *next_vb = next_tree ? Vn : Vc;
            const int next_key0 = next_tree ? (inext - nA) * kBlock : k_begin + inext * kBlock;
            const int next_end = next_tree ? tree_end : k_end;
            const int tile0 = cur_key0 + wave * G::kTileKeys;
            // Lane ids re-read through an opaque copy: the LDS addresses derived from them are then
            // recomputed in each iteration (one or two ALU operations) instead of being kept in
            // registers across the loop, where the larger variants would park them in scratch memory
            // and wait for ALL loads in flight on every reload.
            int r16_l = r16, lane_l = lane;
            asm volatile("" : "+v"(r16_l), "+v"(lane_l));

            // K registers -> own LDS tile (K swizzle); then fetch the next block's K.  The prefetch
            // is issued after the last block too (and ignored): a branch around it would make the
            // compiler wait for all loads in flight wherever it waits for one of them.
            if constexpr (ROPE) {
                if (cur_tree) {
                    // packed keys: rotate at the key's position.  The partner chunk of the same row sits
                    // kHalfChunks lanes away; rows past the end were redirected to the last packed key and
                    // take its position.  The rotated rows also go to a.k_rot (what a cache stores).
                    const int chunk = lane_l % G::kChunks;
#pragma unroll
                    for (int s = 0; s < G::kLoads; ++s) {
                        const int key = tile0 + lane_l / G::kChunks + s * G::kRowsPerLoad;
                        const int key_eff = min(key, tree_end - 1);
                        uint4 pr;
                        pr.x = __shfl_xor(kreg[s].x, kHalfChunks, 64); pr.y = __shfl_xor(kreg[s].y, kHalfChunks, 64);
                        pr.z = __shfl_xor(kreg[s].z, kHalfChunks, 64); pr.w = __shfl_xor(kreg[s].w, kHalfChunks, 64);
                        const int pos = clampi(a.position_ids[(size_t)b * a.N + key_eff], 0, a.max_pos - 1);
                        const float *ct = a.cos_tab + (size_t)pos * (D / 2) + (chunk & (kHalfChunks - 1)) * 8;
                        const float *st = a.sin_tab + (size_t)pos * (D / 2) + (chunk & (kHalfChunks - 1)) * 8;
                        float cs[8], sn[8];
#pragma unroll
                        for (int e = 0; e < 8; ++e) { cs[e] = ct[e]; sn[e] = st[e]; }
                        kreg[s] = rope8<T>(kreg[s], pr, cs, sn, chunk < kHalfChunks);
                        if (a.k_rot != nullptr && key < tree_end)
                            *reinterpret_cast<uint4 *>(static_cast<unsigned char *>(a.k_rot) + ((size_t)bh * a.N + key) * G::kRowBytes + chunk * 16) = kreg[s];
                    }
                }
            }
#pragma unroll
            for (int s = 0; s < G::kLoads; ++s) *reinterpret_cast<uint4 *>(my_tile + k_wr(s)) = kreg[s];
            int pid_cur_next = 0, t0_next = 0;
            if (PAGED && !next_tree) {
                // page of the tile fetched now (looked up one iteration ago), and the lookup for the
                // block after it
                pid_cur_next = pid_next;
                t0_next = ctx_tile_first(next_key0, next_end);
                if (inext + 1 < nA) pid_next = page_of(ctx_tile_first(next_key0 + kBlock, next_end));
                load_tile_paged(Kc, pid_cur_next, t0_next, next_end, kreg);
            } else {
                load_tile(next_kb, next_key0, next_end, kreg);
            }
            wave_lds_sync();

            // S^T tile pair: keys (16 mt + r) x packed rows (16 qt + c), raw (unscaled) scores
            f32x4 sacc[2][NQA];
#pragma unroll
            for (int qt = 0; qt < NQA; ++qt) {
                sacc[0][qt] = f32x4{0.f, 0.f, 0.f, 0.f};
                sacc[1][qt] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int t = 0; t < G::kKSteps; ++t) {
                const vec8 a0 = *reinterpret_cast<const vec8 *>(my_tile + kq_rd(t));
                const vec8 a1 = *reinterpret_cast<const vec8 *>(my_tile + kq_rd(t) + 16 * G::kRowBytes);
#pragma unroll
                for (int qt = 0; qt < NQA; ++qt) {
                    {
                        const vec8 bq = *reinterpret_cast<const vec8 *>(sQ + kq_rd(t) + qt * 16 * G::kRowBytes);
                        sacc[0][qt] = Elem<T>::mfma(a0, bq, sacc[0][qt]);
                        sacc[1][qt] = Elem<T>::mfma(a1, bq, sacc[1][qt]);
                    }
                }
            }
            if (ib == 0) RD_TR(8);

            // per-row maximum over this wave's 32 keys, in log2 units (score * scale * log2 e).  An
            // interior context tile keeps the raw scores (the scale is folded into the exponent
            // later); a tile with masked or out-of-range keys is scaled here and its dead entries
            // set to -inf.
            const int rem = cur_end - tile0;                       // keys of this tile inside the range
            const bool plain = !cur_tree && rem >= G::kTileKeys && !c_neg;
            if (plain) {
#pragma unroll
                for (int qt = 0; qt < NQA; ++qt) {
                    {
                        float tmax = fmaxf(fmaxf(fmaxf(sacc[0][qt][0], sacc[0][qt][1]), fmaxf(sacc[0][qt][2], sacc[0][qt][3])),
                                           fmaxf(fmaxf(sacc[1][qt][0], sacc[1][qt][1]), fmaxf(sacc[1][qt][2], sacc[1][qt][3])));
                        tmax = quad_max(tmax) * c_abs;
                        if (g == 0) sM[(qt * 16 + r16_l) * NW + wave] = tmax;
                    }
                }
            } else {
                const uint32_t tail = rem >= 32 ? 0xffffffffu : (rem <= 0 ? 0u : ((1u << rem) - 1u));
                const uint32_t tail8 = ((tail >> (4 * g)) & 0xfu) | (((tail >> (16 + 4 * g)) & 0xfu) << 4);
                const int tsh = cur_tree ? 8 * (ib - nA) : 0;
#pragma unroll
                for (int qt = 0; qt < NQA; ++qt) {
                    {
                        // element (mt, i) at bit 4 mt + i; context keys are all visible
                        const uint32_t vq = kVisInLds ? sVis[(wave * NQ + qt) * 64 + lane_l] : vis[qt];
                        const uint32_t bits = (cur_tree ? (vq >> tsh) : 0xffu) & tail8;
                        float tmax = -INFINITY;
#pragma unroll
                        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                const float sv = ((bits >> (4 * mt + i)) & 1u) ? sacc[mt][qt][i] * a.scale_log2e : -INFINITY;
                                sacc[mt][qt][i] = sv;
                                tmax = fmaxf(tmax, sv);
                            }
                        tmax = quad_max(tmax);
                        if (g == 0) sM[(qt * 16 + r16_l) * NW + wave] = tmax;
                    }
                }
            }

            lds_barrier();        // (A) tile maxima of all waves visible
            if (ib == 0) RD_TR(9);

            // V registers -> own LDS tile (V swizzle), replacing K which this wave has consumed
#pragma unroll
            for (int s = 0; s < G::kLoads; ++s) *reinterpret_cast<uint4 *>(my_tile + v_wr(s)) = vreg[s];
            if (PAGED && !next_tree) load_tile_paged(Vc, pid_cur_next, t0_next, next_end, vreg);
            else load_tile(next_vb, next_key0, next_end, vreg);

            // online softmax with the block-wide maximum; P^T to LDS in B-operand layout
#pragma unroll
            for (int qt = 0; qt < NQA; ++qt) {
                {
                    const f32x4 *pm = reinterpret_cast<const f32x4 *>(sM + (qt * 16 + r16_l) * NW);
                    f32x4 mv = pm[0];
                    if (NW == 8) {
                        const f32x4 mv2 = pm[1];
                        mv[0] = fmaxf(mv[0], mv2[0]); mv[1] = fmaxf(mv[1], mv2[1]);
                        mv[2] = fmaxf(mv[2], mv2[2]); mv[3] = fmaxf(mv[3], mv2[3]);
                    }
                    const float mb = fmaxf(fmaxf(mv[0], mv[1]), fmaxf(mv[2], mv[3]));
                    const float m_new = fmaxf(m_run[qt], mb);
                    const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
                    const float alpha = __builtin_amdgcn_exp2f(m_run[qt] - m_safe);
                    m_run[qt] = m_new;
                    float psum = 0.f;
                    vec8 pb;
#pragma unroll
                    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const float e = plain ? __builtin_fmaf(sacc[mt][qt][i], c_abs, -m_safe) : sacc[mt][qt][i] - m_safe;
                            const float pv = __builtin_amdgcn_exp2f(e);
                            psum += pv;
                            pb[4 * mt + i] = (T)pv;
                        }
                    l_run[qt] = l_run[qt] * alpha + psum;
                    *reinterpret_cast<vec8 *>(sP + ((wave * NQ + qt) * 64 + lane_l) * 16) = pb;
                    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {      // the maximum moved for some row
#pragma unroll
                        for (int j = 0; j < kDTW; ++j) oacc[j][qt] *= alpha;
                    }
                }
            }
            lds_barrier();        // (B) V tiles and P^T of all waves visible
            if (ib == 0) RD_TR(10);

            // O^T += V^T P^T over the block's key tiles, for this wave's d-tiles.  Key tiles beyond
            // the range were not loaded (their P^T is zero); only the last block of a range can have them.
            auto pv_tile = [&](int kt) __attribute__((always_inline)) {
                const unsigned char *vt = sKV + kt * G::kTileBytes;
                vec8 aV[kDTW];
#pragma unroll
                for (int j = 0; j < kDTW; ++j) {
                    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(vt + vt_rd(wave * kDTW + j)));
                    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(vt + vt_rd(wave * kDTW + j) + 16 * G::kRowBytes));
                    aV[j] = __builtin_bit_cast(vec8, (s16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                }
#pragma unroll
                for (int qt = 0; qt < NQA; ++qt) {
                    const vec8 pB = *reinterpret_cast<const vec8 *>(sP + ((kt * NQ + qt) * 64 + lane) * 16);
#pragma unroll
                    for (int j = 0; j < kDTW; ++j)
                        oacc[j][qt] = Elem<T>::mfma(aV[j], pB, oacc[j][qt]);
                }
            };
            if (cur_key0 + kBlock <= cur_end) {
#pragma unroll
                for (int kt = 0; kt < NW; ++kt) pv_tile(kt);
            } else {
#pragma unroll 1
                for (int kt = 0; cur_key0 + kt * G::kTileKeys < cur_end; ++kt) pv_tile(kt);
            }
            lds_barrier();        // (C) tiles and P^T free for the next block
            if (ib == 0) RD_TR(2);
        }
    };
    constexpr int kHalf = (NQ + 1) / 2;
    if (NQ > 1 && nqt <= kHalf) block_loop(std::integral_constant<int, kHalf>{});
    else if (NQ == 5 && nqt == 4) block_loop(std::integral_constant<int, NQ == 5 ? 4 : NQ>{});   // five tiles spill; four do not
    else block_loop(std::integral_constant<int, NQ>{});
    RD_TR(3);

    // ---- a head served by this workgroup alone: normalise and write the output -------------------
    if (n_part == 1) {
        float *sL1 = sM;          // [kRows][NW]
#pragma unroll
        for (int qt = 0; qt < NQ; ++qt) {
            const float l = quad_sum(l_run[qt]);
            if (g == 0) sL1[(qt * 16 + r16) * NW + wave] = l;
        }
        lds_barrier();
        T *outp = static_cast<T *>(a.out) + ((size_t)bh * a.N + row0) * D;
#pragma unroll
        for (int qt = 0; qt < NQ; ++qt) {
            const int qrow = qt * 16 + r16;
            if (qrow < Ng) {
                float lsum = sL1[qrow * NW];
#pragma unroll
                for (int w = 1; w < NW; ++w) lsum += sL1[qrow * NW + w];
                const bool keep = qrow < P;                               // rows beyond the packed count are zero
                const float inv = keep ? 1.0f / lsum : 0.f;
#pragma unroll
                for (int j = 0; j < kDTW; ++j) {
                    const f32x4 o = oacc[j][qt];
                    store_out4(outp + (size_t)qrow * D + (wave * kDTW + j) * 16 + 4 * g, keep ? o[0] * inv : 0.f,
                               keep ? o[1] * inv : 0.f, keep ? o[2] * inv : 0.f, keep ? o[3] * inv : 0.f);
                }
            }
        }
        RD_TR(6);
        return;
    }

    // ---- partial state of this key range -> workspace ------------------------------------------
    // Layout of one partial: (m, l) pairs [kRows][2], then the output accumulators exactly as the
    // lanes hold them, [wave][d-tile j][row tile qt][lane][4 floats], so that every wave store
    // (and the merge's loads) covers 1 KB of contiguous memory.
    const size_t unit = (size_t)bh * n_rg + rg;                    // (head, row group): one merge each
    float *part = a.partials + (unit * n_part + split) * kPF;
    const int frag_off = 2 * kRows + wave * kDTW * NQ * 256 + lane * 4;    // + (j*NQ + qt)*256
    float *sL = sM;           // reuse: [NW waves][kRows]
#pragma unroll
    for (int qt = 0; qt < NQ; ++qt) {
        const float l = quad_sum(l_run[qt]);
        if (g == 0) sL[(qt * 16 + r16) * NW + wave] = l;
    }
#pragma unroll
    for (int qt = 0; qt < NQ; ++qt) {
        if (qt * 16 + r16 < P) {                        // lanes whose row is padding neither store nor (in the merge) load
#pragma unroll
            for (int j = 0; j < kDTW; ++j) {
                const f32x4 o = oacc[j][qt];
                st_dev4(part + frag_off + (j * NQ + qt) * 256, o[0], o[1], o[2], o[3]);
            }
        }
    }
    lds_barrier();
    if (wave == 0 && g == 0) {
#pragma unroll
        for (int qt = 0; qt < NQ; ++qt) {
            const int qrow = qt * 16 + r16;
            float lsum = sL[qrow * NW];
#pragma unroll
            for (int w = 1; w < NW; ++w) lsum += sL[qrow * NW + w];
            st_dev2(part + 2 * qrow, m_run[qt], lsum);
        }
    }

    // ---- last workgroup of this (sequence, head) merges and writes the output ---------------------
    // With the XCD-aligned mapping every producer of this head ran on this XCD, so their
    // write-through stores also updated this XCD's L2 and plain (cached, 16-byte) loads see them.
    RD_TR(4);
    const int last = arrive_is_last(a.counters + unit, (uint32_t)n_part);
    RD_TR(5);
    if (last == kNotLast) return;
    const bool cached = (last == kLastClean);
    RD_TR(11);
#ifdef RD_TRACE
    if (tid == 0 && rd_trace_buf) rd_trace_buf[(size_t)blockIdx.x * 16 + 13] = 1000 + last * 10 + xcc_id();
#endif

    // Merge: out[q] = sum_s 2^(m_s - M) O_s[q] / sum_s 2^(m_s - M) l_s[q], M = max_s m_s (log2
    // units).  Each thread merges the accumulator fragments it would own itself, two row tiles at
    // a time; the loads of up to kChunk partials for both are issued together, then consumed (the
    // read of a head's partials by one compute unit is what this phase costs, so it should be a
    // single round trip whenever the partials are few).
    constexpr int kChunk = 6;
    const float *hp = a.partials + unit * n_part * kPF;
    T *outp = static_cast<T *>(a.out) + ((size_t)bh * a.N + row0) * D;
    const int nqt_out = (Ng + 15) >> 4;
#pragma unroll 1
    for (int qt0 = 0; qt0 < nqt_out; qt0 += 2) {
        float M[2], den[2];
        f32x4 acc[2][kDTW];
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            M[u] = -INFINITY;
            den[u] = 0.f;
#pragma unroll
            for (int j = 0; j < kDTW; ++j) acc[u][j] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        if (qt0 < nqt) {
            const bool two = qt0 + 1 < nqt;                                     // uniform
#pragma unroll 1
            for (int s0 = 0; s0 < n_part; s0 += kChunk) {
                float2 ml[2][kChunk];
                f32x4 f[2][kChunk][kDTW];
#pragma unroll
                for (int c = 0; c < kChunk; ++c) {
                    const bool have = s0 + c < n_part;                          // uniform
                    const float *ps = hp + (size_t)(s0 + c) * kPF;
#pragma unroll
                    for (int u = 0; u < 2; ++u) {
                        ml[u][c] = make_float2(-INFINITY, 0.f);                 // absent: weight 2^-inf = 0
#pragma unroll
                        for (int j = 0; j < kDTW; ++j) f[u][c][j] = f32x4{0.f, 0.f, 0.f, 0.f};
                        if (have && (u == 0 || two) && (qt0 + u) * 16 + r16 < P) {
                            const int qt = qt0 + u;
                            const float *pm = ps + 2 * (qt * 16 + r16);
                            const float *pf = ps + frag_off + qt * 256;
                            if (cached) {
                                ml[u][c] = *reinterpret_cast<const float2 *>(pm);
#pragma unroll
                                for (int j = 0; j < kDTW; ++j)
                                    f[u][c][j] = *reinterpret_cast<const f32x4 *>(pf + j * NQ * 256);
                            } else {
                                ml[u][c] = ld_dev2(pm);
#pragma unroll
                                for (int j = 0; j < kDTW; ++j) {
                                    const float2 lo = ld_dev2(pf + j * NQ * 256);
                                    const float2 hi = ld_dev2(pf + j * NQ * 256 + 2);
                                    f[u][c][j] = f32x4{lo.x, lo.y, hi.x, hi.y};
                                }
                            }
                        }
                    }
                }
                if (qt0 == 0 && s0 == 0) RD_TR(12);
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    float Mn = M[u];
#pragma unroll
                    for (int c = 0; c < kChunk; ++c) Mn = fmaxf(Mn, ml[u][c].x);
                    const float Ms = (Mn == -INFINITY) ? 0.f : Mn;
                    const float resc = __builtin_amdgcn_exp2f(M[u] - Ms);
                    den[u] *= resc;
#pragma unroll
                    for (int j = 0; j < kDTW; ++j) acc[u][j] *= resc;
#pragma unroll
                    for (int c = 0; c < kChunk; ++c) {
                        const float w = __builtin_amdgcn_exp2f(ml[u][c].x - Ms);     // 0 for an empty or absent range
                        den[u] += w * ml[u][c].y;
#pragma unroll
                        for (int j = 0; j < kDTW; ++j) acc[u][j] += w * f[u][c][j];
                    }
                    M[u] = Mn;
                }
            }
        }
        if (qt0 == 0) RD_TR(7);
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int qrow = (qt0 + u) * 16 + r16;
            if (qrow < Ng) {
                const bool keep = qrow < P;                               // rows beyond the packed count are zero
                const float inv = keep ? 1.0f / den[u] : 0.f;
#pragma unroll
                for (int j = 0; j < kDTW; ++j) {
                    const int d0 = (wave * kDTW + j) * 16 + 4 * g;
                    store_out4(outp + (size_t)qrow * D + d0, keep ? acc[u][j][0] * inv : 0.f, keep ? acc[u][j][1] * inv : 0.f,
                               keep ? acc[u][j][2] * inv : 0.f, keep ? acc[u][j][3] * inv : 0.f);
                }
            }
        }
    }
    if (tid == 0) a.counters[unit] = 0;   // leave the workspace ready for the next call
    RD_TR(6);
}

template <int D, int NQ, int NW>
static size_t mfma_smem_bytes()
{
    return (size_t)NQ * 16 * Geo<D>::kRowBytes + NW * Geo<D>::kTileBytes + (size_t)NW * NQ * 64 * 16 +
           (size_t)NW * NQ * 16 * sizeof(float) + (size_t)NW * NQ * 64 * sizeof(uint32_t);
}

template <typename T, int D, int NQ, int NW, int TB, bool PAGED, bool ROPE = false>
static int launch_mfma(const AttnArgs &a, hipStream_t stream)
{
    const size_t smem = mfma_smem_bytes<D, NQ, NW>();
    static std::atomic<unsigned long long> configured{0};
    const int st = ensure_dynamic_lds(reinterpret_cast<const void *>(&rd_tree_attn_mfma_kernel<T, D, NQ, NW, TB, PAGED, ROPE>), smem,
                                      configured);
    if (st != RD_OK) return st;
    const size_t wgs = (size_t)a.B * a.H * (a.S + (a.fuse_tree ? 0 : 1)) * a.n_rg;
    if (wgs > 0x7fffffffull) return RD_ERR_UNSUPPORTED;
    const unsigned grid = (unsigned)wgs;
    hipLaunchKernelGGL((rd_tree_attn_mfma_kernel<T, D, NQ, NW, TB, PAGED, ROPE>), dim3(grid), dim3(NW * 64), smem, stream, a);
    return rd_check_launch();
}

// rg_tiles = 16-row tiles per workgroup (the template's NQ); D = 128 kernels exist for 1..5 tiles,
// D = 64 kernels for 1..8 (the plan never asks for more).  Beams with more packed keys than one
// block (N > 32*NW) only occur with row groups, i.e. with kGroupTiles tiles.
template <typename T, int D, int NW, bool PAGED, bool ROPE = false>
static int dispatch_nq(const AttnArgs &a, int rg_tiles, hipStream_t stream)
{
    constexpr int kGroupTiles = D == 128 ? 3 : 4;
    const int tb = (a.N + 32 * NW - 1) / (32 * NW);
    if (tb > 1) {
        if (rg_tiles != kGroupTiles) return RD_ERR_UNSUPPORTED;
        if (tb == 2) return launch_mfma<T, D, kGroupTiles, NW, 2, PAGED, ROPE>(a, stream);
        if constexpr (NW == 4) {
            if (tb == 3) return launch_mfma<T, D, kGroupTiles, 4, 3, PAGED, ROPE>(a, stream);
        }
        return RD_ERR_UNSUPPORTED;
    }
    switch (rg_tiles) {
    case 1: return launch_mfma<T, D, 1, NW, 1, PAGED, ROPE>(a, stream);
    case 2: return launch_mfma<T, D, 2, NW, 1, PAGED, ROPE>(a, stream);
    case 3: return launch_mfma<T, D, 3, NW, 1, PAGED, ROPE>(a, stream);
    case 4: return launch_mfma<T, D, 4, NW, 1, PAGED, ROPE>(a, stream);
    case 5: return launch_mfma<T, D, 5, NW, 1, PAGED, ROPE>(a, stream);
    default: break;
    }
    if constexpr (D == 64) {
        switch (rg_tiles) {
        case 6: return launch_mfma<T, 64, 6, NW, 1, PAGED, ROPE>(a, stream);
        case 7: return launch_mfma<T, 64, 7, NW, 1, PAGED, ROPE>(a, stream);
        case 8: return launch_mfma<T, 64, 8, NW, 1, PAGED, ROPE>(a, stream);
        default: break;
        }
    }
    return RD_ERR_UNSUPPORTED;
}

template <typename T, bool PAGED, bool ROPE = false>
static int tree_attn_mfma(const AttnArgs &a, int D, int waves, int rg_tiles, hipStream_t stream)
{
    if (D == 128)
        return waves == 8 ? dispatch_nq<T, 128, 8, PAGED, ROPE>(a, rg_tiles, stream)
                          : dispatch_nq<T, 128, 4, PAGED, ROPE>(a, rg_tiles, stream);
    return dispatch_nq<T, 64, 4, PAGED, ROPE>(a, rg_tiles, stream);
}

}  // namespace rd
