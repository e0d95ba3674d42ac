// Pieces shared by the bf16 (MFMA) and fp32 tree-attention kernels: the split plan, the
// partial-result workspace layout and the in-kernel combine done by the last workgroup
// of a (sequence, head) to finish.
//
// Work decomposition (flash-decoding style).  The keys a packed row may see are the
// context keys 0..ctx_len-1 plus the packed keys allowed by its mask row (Sec. 3.3).  For
// each (sequence, head) the context keys are cut into S contiguous ranges and the packed
// keys form one more range; one workgroup per range computes, for all packed rows at once,
// a partial softmax state (running max m, sum l, unnormalised output O) and stores it in
// the workspace.  The workgroup that finishes last for that (sequence, head) — found with
// a device-scope counter — merges the S+1 partials, normalises and writes the output, so
// the whole operation is a single launch.
#pragma once
#include "rd_internal.h"

namespace rd {

constexpr int kAttnThreads = 256;
constexpr int kBlockKeys = 128;   // keys handled per workgroup iteration

struct AttnPlan {
    int waves;         // waves per workgroup of the bf16 kernel (4 or 8); a block is 32*waves keys
    int S;             // context splits per (sequence, head)
    int fuse_tree;     // 1: the packed keys are the last block of the last context range, not a range of their own
    int n_part;        // workgroups (and partial results) per head: S, or S + 1 with a separate packed-key range
    int rows_pad;      // packed rows padded to a multiple of 16 (fp32 kernel's partial layout)
    int rg_tiles;      // bf16 kernel: 16-row tiles of packed rows per workgroup (a row group)
    int n_rg;          // bf16 kernel: row groups per (sequence, head); 1 unless N is large
    size_t counters_bytes;
    size_t partial_floats;   // floats per partial: m[rows_pad] + l[rows_pad] + O[rows_pad][D]
    size_t total_bytes;
};

// How many context splits per (sequence, head), and whether the packed keys ride on the last
// context range.  Measured behaviour of the kernel on MI355X that the estimate encodes:
//   * a compute unit streams K/V through this kernel at about 27 GB/s whether it holds one
//     workgroup or two, so the blocks of the workgroups that share a compute unit add up; the
//     launch as a whole cannot exceed about 5.5 TB/s;
//   * workgroups beyond the resident capacity (`slots`) start only as earlier ones retire;
//   * more than one workgroup per head costs a merge: about 3 us of latency plus the partial
//     results written and read back once (at roughly 4 TB/s).
// Long ranges (four blocks or more) take the packed keys as one more block; a head with a single
// such range needs no workspace traffic at all.  S minimises the estimated time.
static inline AttnPlan attn_plan(int B, int H, int N, int D, int Cmax, size_t elem_bytes)
{
    AttnPlan p;
    const long long BH = (long long)B * H;
    const double kv_bytes = 2.0 * (double)BH * Cmax * D * (double)elem_bytes;
    const bool small = kv_bytes < 64e6;          // latency-bound: few blocks per range
    // Packed rows per workgroup: all of them while they fit the register budget (5 row tiles at
    // D = 128, 8 at D = 64); wider beams are cut into row groups of 3 (4) tiles, each a workgroup
    // of its own per key range (K/V are then re-read per group, from L2 mostly).
    const int nq_all = (N + 15) / 16;
    static const int tiles_env = env_int("RD_ATTN_ROWTILES", 0);       // tuning: largest single group
    int nq_max = D == 128 ? 5 : 8;
    const int nq_grp = D == 128 ? 3 : 4;
    if (tiles_env >= nq_grp && tiles_env <= nq_max) nq_max = tiles_env;
    const int nq = elem_bytes == 2 ? (nq_all <= nq_max ? nq_all : nq_grp) : nq_all;
    const int n_rg = elem_bytes == 2 ? (nq_all + nq - 1) / nq : 1;
    // Waves per workgroup: eight for small working sets, and also when the heads (and row groups) alone come
    // to one workgroup per compute unit (129..256 of them) over contexts long enough to take the packed keys
    // along: such a launch has no second workgroup per compute unit to overlap with, and eight waves keep
    // 128 KB of loads in flight per compute unit instead of 64 KB.
    static const int waves_env = env_int("RD_ATTN_WAVES", 0);
    const long long units = BH * n_rg;
    const bool one_per_cu = units > 128 && units <= 256 && (Cmax + 255) / 256 >= 4;
    p.waves = (elem_bytes == 2 && D == 128 && (small || one_per_cu)) ? 8 : 4;
    if (waves_env == 4 || (waves_env == 8 && elem_bytes == 2 && D == 128)) p.waves = waves_env;
    const int block_keys = elem_bytes == 2 ? 32 * p.waves : kBlockKeys;
    const int nblk = (Cmax + block_keys - 1) / block_keys;
    const long long slots = (elem_bytes == 2 && p.waves == 4 && nq <= 5) ? 512 : 256;
    const bool can_fuse = elem_bytes == 2;
    const double blk_bytes = 2.0 * block_keys * D * (double)elem_bytes;      // K and V of one block of one head
    const double t_blk = blk_bytes / 27e9;
    const double t_hbm = (double)BH * nblk * blk_bytes / 5.5e12;
    const double part_bytes = (double)nq * 16 * (2 + D) * sizeof(float);
    int best_S = 1;
    double best_T = 1e30;
    for (int S = 1; S <= nblk && S <= 64; ++S) {
        const int per = (nblk + S - 1) / S;
        const bool fuse = can_fuse && per >= 4;
        const int n_part = S + (fuse ? 0 : 1);
        const long long wg = BH * S * n_rg;
        const long long rounds = wg <= slots ? (wg + 255) / 256 : (wg + slots - 1) / slots * (slots / 256);
        double T = (double)rounds * (per + (fuse ? 1 : 0)) * t_blk;
        if (T < t_hbm) T = t_hbm;
        if (n_part > 1) T += 3e-6 + 2.0 * (double)BH * n_rg * n_part * part_bytes / 4e12;
        if (T < best_T * (1.0 - 1e-9)) { best_T = T; best_S = S; }
    }
    if (p.waves == 8 && one_per_cu && !small) best_S = 1;     // the heads fill the compute units by themselves
    static const int forced = env_int("RD_ATTN_SPLITS", 0);
    if (forced > 0) best_S = forced < nblk ? forced : (nblk > 0 ? nblk : 1);
    p.S = best_S;
    static const int fuse_env = env_int("RD_ATTN_FUSE", -1);
    p.fuse_tree = (can_fuse && nblk > 0 && (nblk + p.S - 1) / p.S >= 4) ? 1 : 0;
    if (fuse_env >= 0 && can_fuse && nblk > 0) p.fuse_tree = fuse_env ? 1 : 0;
    p.n_part = p.S + (p.fuse_tree ? 0 : 1);
    p.rows_pad = (N + 15) / 16 * 16;
    p.rg_tiles = nq;
    p.n_rg = n_rg;
    p.counters_bytes = ((size_t)BH * n_rg * sizeof(unsigned long long) + 255) / 256 * 256;
    // floats per partial: fp32 kernel m[rows_pad] + l[rows_pad] + O[rows_pad][D] per (b,h,part);
    // bf16 kernel the same for the rows of one group, per (b,h,group,part)
    p.partial_floats = elem_bytes == 2 ? (size_t)nq * 16 * (2 + D) : (size_t)p.rows_pad * (2 + D);
    p.total_bytes = p.counters_bytes +
                    (p.n_part > 1 ? (size_t)BH * n_rg * p.n_part * p.partial_floats * sizeof(float) : 0);
    return p;
}

struct AttnArgs {
    const void *q, *k_cache, *v_cache, *k_new, *v_new;
    const int32_t *ctx_len, *n_packed;
    const int32_t *block_table;   // paged cache only: [B, max_pages] page of keys [j*page_size, (j+1)*page_size)
    int page_size, max_pages, n_pages;
    const uint64_t *mask_bits;
    void *out;
    unsigned long long *counters;
    float *partials;
    int B, H, N, Cmax, S, words, rows_pad;
    int n_rg;      // row groups per (sequence, head) (bf16 kernel; each is NQ*16 rows of the template)
    int fuse_tree; // 1: packed keys walked by the workgroup of the last context range (see AttnPlan)
    int xcd_remap; // 1: workgroup i serves XCD i%8's share of the heads (needs B*H % 8 == 0)
    float scale_log2e;
    // rotary embedding fused into the call (rd_tree_attn_rope); unused (null) otherwise
    const int32_t *position_ids;   // [B, N]
    const float *cos_tab, *sin_tab;   // [max_pos, D/2]
    int max_pos;
    void *k_rot;                   // [B,H,N,D] rotated packed keys (output), or null
};

__device__ __forceinline__ int clampi(int x, int lo, int hi) { return x < lo ? lo : (x > hi ? hi : x); }

// Context key range [k_begin, k_end) of split s out of S for a context of C keys: whole
// blocks of block_keys keys, spread as evenly as whole blocks allow.
__device__ __forceinline__ void ctx_range(int C, int S, int s, int block_keys, int *k_begin, int *k_end)
{
    const int nblk = (C + block_keys - 1) / block_keys;
    const int per = (nblk + S - 1) / S;
    const int kb = s * per * block_keys;
    *k_begin = kb < C ? kb : C;
    const int ke = kb + per * block_keys;
    *k_end = ke < C ? ke : C;
}

__device__ __forceinline__ void store_out4(float *dst, float a, float b, float c, float d)
{
    *reinterpret_cast<float4 *>(dst) = make_float4(a, b, c, d);
}
__device__ __forceinline__ void store_out4(__bf16 *dst, float a, float b, float c, float d)
{
    typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
    bf16x4 v;
    v[0] = (__bf16)a; v[1] = (__bf16)b; v[2] = (__bf16)c; v[3] = (__bf16)d;   // round to nearest even
    *reinterpret_cast<bf16x4 *>(dst) = v;
}

__device__ __forceinline__ void store_out4(_Float16 *dst, float a, float b, float c, float d)
{
    typedef __attribute__((ext_vector_type(4))) _Float16 f16x4;
    f16x4 v;
    v[0] = (_Float16)a; v[1] = (_Float16)b; v[2] = (_Float16)c; v[3] = (_Float16)d;   // round to nearest even
    *reinterpret_cast<f16x4 *>(dst) = v;
}

// XCD this workgroup runs on (hardware register XCC_ID).
__device__ __forceinline__ uint32_t xcc_id() { return __builtin_amdgcn_s_getreg((31 << 11) | 20) & 0xfu; }

enum { kNotLast = 0, kLastClean = 1, kLastMixed = 2 };

// Signals that this workgroup's partial is stored (with st_dev*); tells every thread of the
// workgroup whether it arrived last among `expected` for this (sequence, head).  The last arriver
// also learns whether every contributor ran on its own XCD (kLastClean: the partials are then
// current in its L2, which is coherent within an XCD) or not (kLastMixed: it must read them with
// ld_dev*, past its L2, which may still hold an older call's lines).  No assumption is made about
// which XCD a workgroup lands on: the 64-bit word collects, beside the count (bits 0-15), the sum
// (bits 16-31) and the sum of squares (bits 32-63) of the contributors' XCD numbers, and n values
// are all equal to x exactly if their sum is n*x and their sum of squares n*x*x.
__device__ __forceinline__ int arrive_is_last(unsigned long long *counter, uint32_t expected)
{
    __shared__ uint32_t s_last;
    wait_dev_stores();
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");   // waits until this thread's stores are acknowledged
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned long long x = xcc_id();
        const unsigned long long add = 1ull | (x << 16) | ((x * x) << 32);
        const unsigned long long now = __hip_atomic_fetch_add(counter, add, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + add;
        const unsigned long long n = now & 0xffffull;
        const bool same = ((now >> 16) & 0xffffull) == n * x && (now >> 32) == n * x * x;
        s_last = (n == expected) ? (same ? kLastClean : kLastMixed) : kNotLast;
    }
    __syncthreads();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");   // later loads stay after the counter update
    return (int)s_last;
}

// Merge of the S+1 partial softmax states of one (sequence, head) and final store:
// out[p] = sum_s 2^(m_s - M) O_s[p] / sum_s 2^(m_s - M) l_s[p] with M = max_s m_s (scores
// are kept in log2 units).  Rows p >= P are written as zero.  Run by one workgroup.
template <int D, typename OutT>
__device__ __forceinline__ void combine_partials(const float *part /* first partial of this head */,
                                                 int n_part, size_t partial_floats, int rows_pad,
                                                 int P, int N, OutT *out /* [N][D] of this head */)
{
    constexpr int kVecPerRow = D / 4;
    constexpr int kRowsPerPass = kAttnThreads / kVecPerRow;
    const int tid = threadIdx.x;
    const int v = tid % kVecPerRow;
    for (int p = tid / kVecPerRow; p < N; p += kRowsPerPass) {
        float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
        if (p < P) {
            float M = -INFINITY;
            for (int s = 0; s < n_part; ++s) M = fmaxf(M, ld_dev(part + s * partial_floats + p));
            float denom = 0.f;
            for (int s = 0; s < n_part; ++s) {
                const float *ps = part + s * partial_floats;
                const float m = ld_dev(ps + p);
                if (m == -INFINITY) continue;          // that range held no visible key for row p
                const float w = __builtin_amdgcn_exp2f(m - M);
                denom += w * ld_dev(ps + rows_pad + p);
                const float *po = ps + 2 * rows_pad + (size_t)p * D + 4 * v;
                const float2 o01 = ld_dev2(po), o23 = ld_dev2(po + 2);
                a0 += w * o01.x; a1 += w * o01.y; a2 += w * o23.x; a3 += w * o23.y;
            }
            const float inv = 1.0f / denom;
            a0 *= inv; a1 *= inv; a2 *= inv; a3 *= inv;
        }
        store_out4(out + (size_t)p * D + 4 * v, a0, a1, a2, a3);
    }
}

}  // namespace rd
