// rd_tree_attn, bf16 path: tree-masked attention of the packed candidates against the KV
// cache (Sec. 3.3, 3.4) as a split-key flash kernel on the gfx950 matrix cores.
//
// Decoding attention is bound by streaming K and V from HBM (512 bytes per key and head at
// D = 128) while the packed rows (at most 128) are reused for every key, so the kernel is
// organised around the stream:
//   * a workgroup (4 waves) owns a contiguous key range of one (sequence, head) and walks
//     it in blocks of 128 keys; wave w loads rows 32w..32w+31 of the block for K and for V
//     with fully coalesced 16-byte-per-lane loads (a wave instruction covers whole 256-byte
//     rows), one block ahead of the arithmetic, and parks them in LDS;
//   * scores are produced transposed, S^T = K Q^T, with v_mfma_f32_16x16x32_bf16: the wave
//     reads its own K tile back from LDS in the A-operand layout (XOR-swizzled, conflict
//     free) and Q (resident in LDS for the whole kernel) as the B operand;
//   * tree mask (bit test against tree_mask_bits) and range limits are applied to the
//     accumulators in registers; the four waves exchange their per-row tile maxima through
//     LDS so the block has one running maximum per packed row (online softmax, log2 units);
//   * the probabilities, rounded to bf16, are written to LDS already in B-operand layout;
//     the accumulator layout of S^T makes each lane's eight values exactly one B operand
//     once the 32 keys of a tile are taken in the order (4g+i, 16+4g+i);
//   * O^T = V^T P^T: wave w owns d-tiles 2w and 2w+1 (D = 128) for all 128 keys of the
//     block; the A operand V^T needs eight keys of one column per lane, which
//     ds_read_b64_tr_b16 (LDS transpose read) delivers from the row-major V tiles, taken in
//     the same key order.  The output accumulators therefore need no cross-wave reduction.
//   * the partial state goes to the workspace and the last workgroup of the head merges.
#include "rd_attn_common.h"

namespace rd {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;

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

template <int D, int NQ>
__global__ __launch_bounds__(kAttnThreads, 2) void rd_tree_attn_bf16_kernel(AttnArgs a)
{
    using G = Geo<D>;
    constexpr int kRows = NQ * 16;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char *sQ = smem;                                   // [kRows][kRowBytes]
    unsigned char *sKV = sQ + kRows * G::kRowBytes;             // 4 tiles [32][kRowBytes]
    unsigned char *sP = sKV + 4 * G::kTileBytes;                // [4 kt][NQ][64 lanes] x 16 B
    float *sM = reinterpret_cast<float *>(sP + 4 * NQ * 64 * 16);   // [4 waves][kRows]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int r16 = lane & 15;
    const int g = lane >> 4;

    const int n_part = a.S + 1;
    const int bh = blockIdx.x / n_part;
    const int split = blockIdx.x % n_part;
    const int b = bh / a.H;
    const int C = clampi(a.ctx_len[b], 0, a.Cmax);
    const int P = clampi(a.n_packed[b], 0, a.N);
    const bool is_tree = (split == a.S);

    int k_begin, k_end;
    const __bf16 *Kb, *Vb;
    if (is_tree) {
        k_begin = 0;
        k_end = P;
        Kb = static_cast<const __bf16 *>(a.k_new) + (size_t)bh * a.N * D;
        Vb = static_cast<const __bf16 *>(a.v_new) + (size_t)bh * a.N * D;
    } else {
        ctx_range(C, a.S, split, &k_begin, &k_end);
        Kb = static_cast<const __bf16 *>(a.k_cache) + (size_t)bh * a.Cmax * D;
        Vb = static_cast<const __bf16 *>(a.v_cache) + (size_t)bh * a.Cmax * D;
    }

    // ---- this wave's slice of a block: guarded, coalesced loads into registers -------------
    uint4 kreg[G::kLoads], vreg[G::kLoads];
    const int ld_row = lane / G::kChunks;        // row within one load
    const int ld_chunk = lane % G::kChunks;
    auto load_tile = [&](const __bf16 *base, int tile0, uint4 (&reg)[G::kLoads]) {
#pragma unroll
        for (int s = 0; s < G::kLoads; ++s) {
            const int key = tile0 + s * G::kRowsPerLoad + ld_row;
            reg[s] = (key < k_end) ? ldg16(base + (size_t)key * D + ld_chunk * 8) : make_uint4(0, 0, 0, 0);
        }
    };
    load_tile(Kb, k_begin + wave * G::kTileKeys, kreg);
    load_tile(Vb, k_begin + wave * G::kTileKeys, vreg);

    // ---- Q of this head into LDS (rows >= P zeroed) ------------------------------------------
    {
        const __bf16 *Qb = static_cast<const __bf16 *>(a.q) + (size_t)bh * a.N * D;
        constexpr int kRowsPerPass = kAttnThreads / G::kChunks;
        const int c = tid % G::kChunks;
#pragma unroll
        for (int r0 = 0; r0 < kRows; r0 += kRowsPerPass) {
            const int row = r0 + tid / G::kChunks;
            if (row < kRows) {
                const uint4 v = (row < P) ? ldg16(Qb + (size_t)row * D + c * 8) : make_uint4(0, 0, 0, 0);
                *reinterpret_cast<uint4 *>(sQ + row * G::kRowBytes + kswz<D>(row, c) * 16) = v;
            }
        }
    }

    // ---- tree mask rows of the packed rows this lane scores (row 16*qt + r16) ------------------
    uint64_t mw[NQ][2];
#pragma unroll
    for (int qt = 0; qt < NQ; ++qt) {
        mw[qt][0] = 0;
        mw[qt][1] = 0;
        const int qrow = qt * 16 + r16;
        if (is_tree && qrow < P) {
            const uint64_t *mrow = a.mask_bits + ((size_t)b * a.N + qrow) * a.words;
            mw[qt][0] = mrow[0];
            if (a.words > 1) mw[qt][1] = mrow[1];
        }
    }

    float m_run[NQ], l_run[NQ];
    f32x4 oacc[G::kDTilesPerWave][NQ];
#pragma unroll
    for (int qt = 0; qt < NQ; ++qt) {
        m_run[qt] = -INFINITY;
        l_run[qt] = 0.f;
#pragma unroll
        for (int j = 0; j < G::kDTilesPerWave; ++j) oacc[j][qt] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    unsigned char *my_tile = sKV + wave * G::kTileBytes;

    for (int blk0 = k_begin; blk0 < k_end; blk0 += kBlockKeys) {
        const int tile0 = blk0 + wave * G::kTileKeys;
        const bool more = blk0 + kBlockKeys < k_end;

        // K registers -> own LDS tile (K swizzle); then fetch the next block's K
#pragma unroll
        for (int s = 0; s < G::kLoads; ++s) {
            const int row = s * G::kRowsPerLoad + ld_row;
            *reinterpret_cast<uint4 *>(my_tile + row * G::kRowBytes + kswz<D>(row, ld_chunk) * 16) = kreg[s];
        }
        if (more) load_tile(Kb, tile0 + kBlockKeys, kreg);
        __syncthreads();      // K tile (and, first time round, Q) visible

        // S^T tile pair: keys (16 mt + r) x packed rows (16 qt + c)
        f32x4 sacc[2][NQ];
#pragma unroll
        for (int qt = 0; qt < NQ; ++qt) {
            sacc[0][qt] = f32x4{0.f, 0.f, 0.f, 0.f};
            sacc[1][qt] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int t = 0; t < G::kKSteps; ++t) {
            const int c = 4 * t + g;
            const bf16x8 a0 = *reinterpret_cast<const bf16x8 *>(my_tile + r16 * G::kRowBytes + kswz<D>(r16, c) * 16);
            const bf16x8 a1 = *reinterpret_cast<const bf16x8 *>(my_tile + (16 + r16) * G::kRowBytes + kswz<D>(16 + r16, c) * 16);
#pragma unroll
            for (int qt = 0; qt < NQ; ++qt) {
                const int qrow = qt * 16 + r16;
                const bf16x8 bq = *reinterpret_cast<const bf16x8 *>(sQ + qrow * G::kRowBytes + kswz<D>(qrow, c) * 16);
                sacc[0][qt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, bq, sacc[0][qt], 0, 0, 0);
                sacc[1][qt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, bq, sacc[1][qt], 0, 0, 0);
            }
        }

        // mask + scale (log2 units) + per-row maximum over this wave's 32 keys
#pragma unroll
        for (int qt = 0; qt < NQ; ++qt) {
            float tmax = -INFINITY;
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int key = tile0 + 16 * mt + 4 * g + i;
                    bool ok = key < k_end;
                    if (is_tree) ok = ok && ((((key & 64) ? mw[qt][1] : mw[qt][0]) >> (key & 63)) & 1ull);
                    const float s = ok ? sacc[mt][qt][i] * a.scale_log2e : -INFINITY;
                    sacc[mt][qt][i] = s;
                    tmax = fmaxf(tmax, s);
                }
            tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
            tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
            if (g == 0) sM[wave * kRows + qt * 16 + r16] = tmax;
        }

        // V registers -> own LDS tile (V swizzle), replacing K which this wave has consumed
        __syncthreads();      // every wave is done reading its K tile
#pragma unroll
        for (int s = 0; s < G::kLoads; ++s) {
            const int row = s * G::kRowsPerLoad + ld_row;
            *reinterpret_cast<uint4 *>(my_tile + row * G::kRowBytes + vswz<D>(row, ld_chunk) * 16) = vreg[s];
        }
        if (more) load_tile(Vb, tile0 + kBlockKeys, vreg);

        // online softmax with the block-wide maximum; P^T to LDS in B-operand layout
#pragma unroll
        for (int qt = 0; qt < NQ; ++qt) {
            const int qrow = qt * 16 + r16;
            float mb = fmaxf(fmaxf(sM[qrow], sM[kRows + qrow]), fmaxf(sM[2 * kRows + qrow], sM[3 * kRows + qrow]));
            const float m_new = fmaxf(m_run[qt], mb);
            const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
            const float alpha = __builtin_amdgcn_exp2f(m_run[qt] - m_safe);
            m_run[qt] = m_new;
            float psum = 0.f;
            bf16x8 pb;
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float p = __builtin_amdgcn_exp2f(sacc[mt][qt][i] - m_safe);
                    psum += p;
                    pb[4 * mt + i] = (__bf16)p;
                }
            l_run[qt] = l_run[qt] * alpha + psum;
            *reinterpret_cast<bf16x8 *>(sP + ((wave * NQ + qt) * 64 + lane) * 16) = pb;
#pragma unroll
            for (int j = 0; j < G::kDTilesPerWave; ++j) oacc[j][qt] *= alpha;
        }
        __syncthreads();      // V tiles and P^T of all four waves visible

        // O^T += V^T P^T over the block's four key tiles, for this wave's d-tiles
#pragma unroll
        for (int kt = 0; kt < 4; ++kt) {
            if (blk0 + kt * G::kTileKeys >= k_end) break;     // tile beyond the range: P^T is zero
            const unsigned char *vt = sKV + kt * G::kTileBytes;
            bf16x8 pB[NQ];
#pragma unroll
            for (int qt = 0; qt < NQ; ++qt)
                pB[qt] = *reinterpret_cast<const bf16x8 *>(sP + ((kt * NQ + qt) * 64 + lane) * 16);
#pragma unroll
            for (int j = 0; j < G::kDTilesPerWave; ++j) {
                const int dt = wave * G::kDTilesPerWave + j;
                const int c = 2 * dt + ((r16 & 3) >> 1);
                const int ra = 4 * g + (r16 >> 2);
                const int rb = 16 + ra;
                const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) s16x4 *)(vt + ra * G::kRowBytes + vswz<D>(ra, c) * 16 + (r16 & 1) * 8));
                const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) s16x4 *)(vt + rb * G::kRowBytes + vswz<D>(rb, c) * 16 + (r16 & 1) * 8));
                typedef __attribute__((ext_vector_type(8))) short s16x8;
                const s16x8 av = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                const bf16x8 aV = __builtin_bit_cast(bf16x8, av);
#pragma unroll
                for (int qt = 0; qt < NQ; ++qt)
                    oacc[j][qt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(aV, pB[qt], oacc[j][qt], 0, 0, 0);
            }
        }
        __syncthreads();      // tiles and P^T free for the next block
    }

    // ---- partial state of this key range -> workspace ------------------------------------------
    float *part = a.partials + ((size_t)bh * n_part + split) * ((size_t)a.rows_pad * (2 + D));
    float *sL = sM;           // reuse: [4 waves][kRows]
#pragma unroll
    for (int qt = 0; qt < NQ; ++qt) {
        float l = l_run[qt];
        l += __shfl_xor(l, 16, 64);
        l += __shfl_xor(l, 32, 64);
        if (g == 0) sL[wave * kRows + qt * 16 + r16] = l;
    }
    __syncthreads();
    if (wave == 0) {
#pragma unroll
        for (int qt = 0; qt < NQ; ++qt) {
            const int qrow = qt * 16 + r16;
            if (g == 0 && qrow < P) {
                part[qrow] = m_run[qt];
                part[a.rows_pad + qrow] = sL[qrow] + sL[kRows + qrow] + sL[2 * kRows + qrow] + sL[3 * kRows + qrow];
            }
        }
    }
#pragma unroll
    for (int qt = 0; qt < NQ; ++qt) {
        const int qrow = qt * 16 + r16;
        if (qrow < P) {
#pragma unroll
            for (int j = 0; j < G::kDTilesPerWave; ++j) {
                const int d0 = (wave * G::kDTilesPerWave + j) * 16 + 4 * g;
                const f32x4 o = oacc[j][qt];
                *reinterpret_cast<float4 *>(part + 2 * a.rows_pad + (size_t)qrow * D + d0) =
                    make_float4(o[0], o[1], o[2], o[3]);
            }
        }
    }

    // ---- last workgroup of this (sequence, head) merges and writes the output ---------------------
    if (arrive_is_last(a.counters + bh, (uint32_t)n_part)) {
        combine_partials<D, __bf16>(a.partials + (size_t)bh * n_part * ((size_t)a.rows_pad * (2 + D)), n_part,
                                    (size_t)a.rows_pad * (2 + D), a.rows_pad, P, a.N,
                                    static_cast<__bf16 *>(a.out) + (size_t)bh * a.N * D);
        if (tid == 0) a.counters[bh] = 0;     // leave the workspace ready for the next call
    }
}

template <int D, int NQ>
static size_t bf16_smem_bytes()
{
    return (size_t)NQ * 16 * Geo<D>::kRowBytes + 4 * Geo<D>::kTileBytes + (size_t)4 * NQ * 64 * 16 +
           (size_t)4 * NQ * 16 * sizeof(float);
}

template <int D, int NQ>
static int launch_bf16(const AttnArgs &a, hipStream_t stream)
{
    const size_t smem = bf16_smem_bytes<D, NQ>();
    static bool configured = false;          // raising the dynamic LDS limit is per kernel, once
    if (!configured) {
        if (hipFuncSetAttribute(reinterpret_cast<const void *>(&rd_tree_attn_bf16_kernel<D, NQ>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess)
            return RD_ERR_HIP;
        configured = true;
    }
    const unsigned grid = (unsigned)((size_t)a.B * a.H * (a.S + 1));
    hipLaunchKernelGGL((rd_tree_attn_bf16_kernel<D, NQ>), dim3(grid), dim3(kAttnThreads), smem, stream, a);
    return rd_check_launch();
}

template <int D>
static int dispatch_nq(const AttnArgs &a, hipStream_t stream)
{
    switch ((a.N + 15) / 16) {
    case 1: return launch_bf16<D, 1>(a, stream);
    case 2: return launch_bf16<D, 2>(a, stream);
    case 3: return launch_bf16<D, 3>(a, stream);
    case 4: return launch_bf16<D, 4>(a, stream);
    case 5: return launch_bf16<D, 5>(a, stream);
    case 6: return launch_bf16<D, 6>(a, stream);
    case 7: return launch_bf16<D, 7>(a, stream);
    case 8: return launch_bf16<D, 8>(a, stream);
    default: return RD_ERR_UNSUPPORTED;
    }
}

int tree_attn_bf16(const AttnArgs &a, int D, hipStream_t stream)
{
    return D == 128 ? dispatch_nq<128>(a, stream) : dispatch_nq<64>(a, stream);
}

}  // namespace rd
