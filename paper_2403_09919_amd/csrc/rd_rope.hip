// rd_rope: rotary position embedding of the packed candidates' queries and keys, with the
// positions rd_dedup produced (position_ids = ctx_len + depth).  The paper's LLMs (Vicuna, Sec. 4)
// are LLaMA-family models, whose attention rotates q and k before the scores; pairing convention
// "rotate half" (element i with element i + D/2).  Elementwise work on a few hundred KB: each
// thread rotates one pair of 16-byte chunks (eight pairs) of q and of k, fp32 arithmetic, one
// rounding to the storage type.
#include "rd_internal.h"

namespace {

constexpr int kRopeThreads = 256;

template <typename T> struct Vec8;       // eight elements of the storage type = 16 bytes (fp32: two of them)
template <> struct Vec8<__bf16> { typedef __attribute__((ext_vector_type(8))) __bf16 type; };
template <> struct Vec8<_Float16> { typedef __attribute__((ext_vector_type(8))) _Float16 type; };
template <> struct Vec8<float> { typedef __attribute__((ext_vector_type(8))) float type; };

// One work item = (b, h, p, chunk c < D/16): elements 8c..8c+7 and their partners D/2 + 8c..+7.
template <typename T, int D>
__global__ __launch_bounds__(kRopeThreads) void rd_rope_kernel(
    T *__restrict__ q, T *__restrict__ k, const int32_t *__restrict__ position_ids,
    const int32_t *__restrict__ n_packed, const float *__restrict__ cos_tab, const float *__restrict__ sin_tab,
    int max_pos, int H, int N, long long total)
{
    typedef typename Vec8<T>::type vec8;
    constexpr int kHalf = D / 2, kChunks = kHalf / 8;
    const long long item = (long long)blockIdx.x * kRopeThreads + threadIdx.x;
    if (item >= total) return;
    const int c = (int)(item % kChunks);
    const long long row = item / kChunks;                  // (b*H + h)*N + p
    const int p = (int)(row % N);
    const int b = (int)(row / ((long long)N * H));
    int P = n_packed[b];
    P = P < 0 ? 0 : (P > N ? N : P);
    if (p >= P) return;
    int pos = position_ids[(size_t)b * N + p];
    pos = pos < 0 ? 0 : (pos > max_pos - 1 ? max_pos - 1 : pos);
    const float *ct = cos_tab + (size_t)pos * kHalf + 8 * c;
    const float *st = sin_tab + (size_t)pos * kHalf + 8 * c;
    float cs[8], sn[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) { cs[i] = ct[i]; sn[i] = st[i]; }
    const size_t off = (size_t)row * D + 8 * c;
#pragma unroll
    for (int which = 0; which < 2; ++which) {
        T *x = which ? k : q;
        if (x == nullptr) continue;
        const vec8 lo = *reinterpret_cast<const vec8 *>(x + off);
        const vec8 hi = *reinterpret_cast<const vec8 *>(x + off + kHalf);
        vec8 ylo, yhi;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float a = (float)lo[i], bb = (float)hi[i];
            // each product is rounded to fp32 before the sum (no fused multiply-add), and the sum is
            // an fp32 value before it is rounded to the storage type: the empty asm keeps the compiler
            // from folding the sum into a mixed-precision instruction that rounds it to fp16 directly
            // (v_fma_mixlo_f16), which differs from this definition in rare double-rounding cases
            float rlo = __fsub_rn(__fmul_rn(a, cs[i]), __fmul_rn(bb, sn[i]));
            float rhi = __fadd_rn(__fmul_rn(bb, cs[i]), __fmul_rn(a, sn[i]));
            asm volatile("" : "+v"(rlo), "+v"(rhi));
            ylo[i] = (T)rlo;
            yhi[i] = (T)rhi;
        }
        *reinterpret_cast<vec8 *>(x + off) = ylo;
        *reinterpret_cast<vec8 *>(x + off + kHalf) = yhi;
    }
}

template <typename T>
int launch_rope(void *q, void *k, const int32_t *position_ids, const int32_t *n_packed, const float *cos_tab,
                const float *sin_tab, int max_pos, int B, int H, int N, int D, hipStream_t stream)
{
    const long long total = (long long)B * H * N * (D / 16);
    const long long blocks = (total + kRopeThreads - 1) / kRopeThreads;
    if (blocks > 0x7fffffffll) return RD_ERR_UNSUPPORTED;
    if (D == 128)
        hipLaunchKernelGGL((rd_rope_kernel<T, 128>), dim3((unsigned)blocks), dim3(kRopeThreads), 0, stream,
                           static_cast<T *>(q), static_cast<T *>(k), position_ids, n_packed, cos_tab, sin_tab, max_pos, H, N, total);
    else
        hipLaunchKernelGGL((rd_rope_kernel<T, 64>), dim3((unsigned)blocks), dim3(kRopeThreads), 0, stream,
                           static_cast<T *>(q), static_cast<T *>(k), position_ids, n_packed, cos_tab, sin_tab, max_pos, H, N, total);
    return rd_check_launch();
}

}  // namespace

extern "C" int rd_rope(void *q, void *k_new, const int32_t *position_ids, const int32_t *n_packed,
                       const float *cos_tab, const float *sin_tab, int max_pos,
                       int B, int H, int N, int D, rd_dtype dt, void *stream)
{
    if (B <= 0 || H <= 0 || N <= 0 || max_pos <= 0) return RD_ERR_INVALID_ARG;
    if (dt != RD_F32 && dt != RD_BF16 && dt != RD_F16) return RD_ERR_UNSUPPORTED;
    if ((D != 64 && D != 128) || N > RD_MAX_N) return RD_ERR_UNSUPPORTED;
    if ((!q && !k_new) || !position_ids || !n_packed || !cos_tab || !sin_tab) return RD_ERR_INVALID_ARG;
    if (!rd_aligned(q, 32) || !rd_aligned(k_new, 32) || !rd_aligned(cos_tab, 4) || !rd_aligned(sin_tab, 4))
        return RD_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    if (dt == RD_BF16) return launch_rope<__bf16>(q, k_new, position_ids, n_packed, cos_tab, sin_tab, max_pos, B, H, N, D, s);
    if (dt == RD_F16) return launch_rope<_Float16>(q, k_new, position_ids, n_packed, cos_tab, sin_tab, max_pos, B, H, N, D, s);
    return launch_rope<float>(q, k_new, position_ids, n_packed, cos_tab, sin_tab, max_pos, B, H, N, D, s);
}
