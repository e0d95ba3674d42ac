// rd_tree_attn, fp32 path: the same split-key scheme as the bf16 kernel with plain fp32
// FMA arithmetic (no matrix cores), for fp32 Q/K/V where results must hold to ~1e-6.
//
// A workgroup handles 16 packed rows of one (sequence, head) over one key range; wave w
// owns rows 4w..4w+3 completely (scores, softmax state, output), so waves only meet at
// the barriers that recycle the K/V tiles in LDS.  Per 64-key tile: lane = key for the
// scores (K rows padded by one float so the 64 lanes hit 64 banks), lane = output column
// for the value product (probabilities are broadcast reads).
#include "rd_attn_common.h"

namespace rd {

constexpr int kF32TileKeys = 64;
constexpr int kF32Rows = 16;

template <int D>
__global__ __launch_bounds__(kAttnThreads) void rd_tree_attn_f32_kernel(AttnArgs a, int row_groups)
{
    constexpr int kKStride = D + 1;
    constexpr int kCols = D / 64;                        // output columns per lane
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float *sQ = reinterpret_cast<float *>(smem);         // [16][D]
    float *sK = sQ + kF32Rows * D;                       // [64][D+1]
    float *sV = sK + kF32TileKeys * kKStride;            // [64][D]
    float *sS = sV + kF32TileKeys * D;                   // [16][64]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;

    const int n_part = a.S + 1;
    const int rg = blockIdx.x % row_groups;
    const int split = (blockIdx.x / row_groups) % n_part;
    const int bh = blockIdx.x / (row_groups * n_part);
    const int b = bh / a.H;
    const int C = clampi(a.ctx_len[b], 0, a.Cmax);
    const int P = clampi(a.n_packed[b], 0, a.N);
    const bool is_tree = (split == a.S);
    const int row0 = rg * kF32Rows;

    int k_begin, k_end;
    const float *Kb, *Vb;
    if (is_tree) {
        k_begin = 0;
        k_end = P;
        Kb = static_cast<const float *>(a.k_new) + (size_t)bh * a.N * D;
        Vb = static_cast<const float *>(a.v_new) + (size_t)bh * a.N * D;
    } else {
        ctx_range(C, a.S, split, kBlockKeys, &k_begin, &k_end);
        Kb = static_cast<const float *>(a.k_cache) + (size_t)bh * a.Cmax * D;
        Vb = static_cast<const float *>(a.v_cache) + (size_t)bh * a.Cmax * D;
    }
    if (row0 >= P) k_end = k_begin;                      // nothing to score: empty partial

    {   // Q rows of this group (rows >= P zeroed)
        const float *Qb = static_cast<const float *>(a.q) + (size_t)bh * a.N * D;
        for (int i = tid; i < kF32Rows * D; i += kAttnThreads) {
            const int row = row0 + i / D;
            sQ[i] = (row < P) ? Qb[(size_t)row * D + (i % D)] : 0.f;
        }
    }

    float m_run[4], l_run[4], o[4][kCols];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        m_run[r] = -INFINITY;
        l_run[r] = 0.f;
#pragma unroll
        for (int c = 0; c < kCols; ++c) o[r][c] = 0.f;
    }

    for (int t0 = k_begin; t0 < k_end; t0 += kF32TileKeys) {
        __syncthreads();                                 // previous tile fully consumed (and Q stored)
        for (int i = tid; i < kF32TileKeys * (D / 4); i += kAttnThreads) {
            const int kr = i / (D / 4), c4 = (i % (D / 4)) * 4;
            const int key = t0 + kr;
            float4 kv = make_float4(0.f, 0.f, 0.f, 0.f), vv = kv;
            if (key < k_end) {
                kv = *reinterpret_cast<const float4 *>(Kb + (size_t)key * D + c4);
                vv = *reinterpret_cast<const float4 *>(Vb + (size_t)key * D + c4);
            }
            float *kd = sK + kr * kKStride + c4;
            kd[0] = kv.x; kd[1] = kv.y; kd[2] = kv.z; kd[3] = kv.w;
            *reinterpret_cast<float4 *>(sV + kr * D + c4) = vv;
        }
        __syncthreads();

        // scores of this wave's four rows against key t0 + lane
        float s[4] = {0.f, 0.f, 0.f, 0.f};
        const float *krow = sK + lane * kKStride;
        const float *q0 = sQ + (wave * 4) * D;
#pragma unroll 8
        for (int d = 0; d < D; ++d) {
            const float kv = krow[d];
            s[0] = fmaf(q0[d], kv, s[0]);
            s[1] = fmaf(q0[D + d], kv, s[1]);
            s[2] = fmaf(q0[2 * D + d], kv, s[2]);
            s[3] = fmaf(q0[3 * D + d], kv, s[3]);
        }
        const int key = t0 + lane;
        float alpha[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            bool ok = key < k_end;
            if (is_tree) {                               // packed keys t0 .. t0+63 are mask word t0/64 of the row
                const int qrow = row0 + wave * 4 + r;
                const uint64_t mw = qrow < P ? a.mask_bits[((size_t)b * a.N + qrow) * a.words + (t0 >> 6)] : 0ull;
                ok = ok && ((mw >> lane) & 1ull);
            }
            const float sv = ok ? s[r] * a.scale_log2e : -INFINITY;
            float tmax = sv;
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) tmax = fmaxf(tmax, __shfl_xor(tmax, off, 64));
            const float m_new = fmaxf(m_run[r], tmax);
            const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
            alpha[r] = __builtin_amdgcn_exp2f(m_run[r] - m_safe);
            m_run[r] = m_new;
            const float p = __builtin_amdgcn_exp2f(sv - m_safe);
            float psum = p;
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) psum += __shfl_xor(psum, off, 64);
            l_run[r] = l_run[r] * alpha[r] + psum;
            sS[(wave * 4 + r) * kF32TileKeys + lane] = p;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __builtin_amdgcn_wave_barrier();                 // sS rows are private to this wave
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");

#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int c = 0; c < kCols; ++c) o[r][c] *= alpha[r];
        const float *ps = sS + (wave * 4) * kF32TileKeys;
        for (int k = 0; k < kF32TileKeys; ++k) {
#pragma unroll
            for (int c = 0; c < kCols; ++c) {
                const float vv = sV[k * D + c * 64 + lane];
#pragma unroll
                for (int r = 0; r < 4; ++r) o[r][c] = fmaf(ps[r * kF32TileKeys + k], vv, o[r][c]);
            }
        }
    }

    const size_t pf = (size_t)a.rows_pad * (2 + D);
    float *part = a.partials + ((size_t)bh * n_part + split) * pf;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int qrow = row0 + wave * 4 + r;
        if (qrow < P) {
            if (lane == 0) {
                st_dev(part + qrow, m_run[r]);
                st_dev(part + a.rows_pad + qrow, l_run[r]);
            }
#pragma unroll
            for (int c = 0; c < kCols; ++c) st_dev(part + 2 * a.rows_pad + (size_t)qrow * D + c * 64 + lane, o[r][c]);
        }
    }

    if (arrive_is_last(a.counters + bh, (uint32_t)(n_part * row_groups)) != kNotLast) {
        combine_partials<D, float>(a.partials + (size_t)bh * n_part * pf, n_part, pf, a.rows_pad, P, a.N,
                                   static_cast<float *>(a.out) + (size_t)bh * a.N * D);
        if (tid == 0) a.counters[bh] = 0;
    }
}

template <int D>
static int launch_f32(const AttnArgs &a, hipStream_t stream)
{
    const size_t smem = sizeof(float) * ((size_t)kF32Rows * D + (size_t)kF32TileKeys * (D + 1) +
                                         (size_t)kF32TileKeys * D + (size_t)kF32Rows * kF32TileKeys);
    static std::atomic<unsigned long long> configured{0};
    const int st = ensure_dynamic_lds(reinterpret_cast<const void *>(&rd_tree_attn_f32_kernel<D>), smem, configured);
    if (st != RD_OK) return st;
    const int row_groups = a.rows_pad / kF32Rows;
    const size_t wgs = (size_t)a.B * a.H * (a.S + 1) * row_groups;
    if (wgs > 0x7fffffffull) return RD_ERR_UNSUPPORTED;
    const unsigned grid = (unsigned)wgs;
    hipLaunchKernelGGL((rd_tree_attn_f32_kernel<D>), dim3(grid), dim3(kAttnThreads), smem, stream, a, row_groups);
    return rd_check_launch();
}

int tree_attn_f32(const AttnArgs &a, int D, hipStream_t stream)
{
    return D == 128 ? launch_f32<128>(a, stream) : launch_f32<64>(a, stream);
}

}  // namespace rd
