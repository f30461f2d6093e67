// Single-query attention (Eq. 4) over cached ++ regenerated K/V (Eq. 3) for gfx950.
//
// The decode query of each (sequence, head) attends over every context token.  With one query
// per head the work is one pass over K and one over V: ~1 FLOP per byte, so the kernel is an HBM
// streaming kernel and is organised around the loads, not the arithmetic:
//   * The context of a (sequence, head) is two contiguous token segments (the cached rows and
//     the regenerated rows); they are never copied together.
//   * Work is split by bytes, not by (sequence, head): the tokens of all pairs form one line of
//     BH * L positions that is cut into W equal ranges, one per wavefront, with W chosen so that
//     all wavefronts are resident at once.  Every wavefront therefore streams the same number of
//     bytes and they all finish together; there is no partly filled last round of workgroups.
//     A range may cover the end of one pair and the start of the next; for every pair it touches
//     a wavefront emits one un-normalised partial (m, l, o[dh]) at index (wavefront + pair), which
//     is unique, and makes the partials of one pair a contiguous run.  A second small kernel
//     merges the run of every pair by log-sum-exp.  Wavefronts never talk to each other: no LDS,
//     no barrier.
//   * A wavefront consumes 64 tokens at a time.  dh/8 lanes cover one row with 16-byte loads, so
//     every load instruction of a wavefront reads whole, consecutive rows (1 KiB contiguous), and
//     all K and V loads of the 64 tokens are issued before the first use.
//   * q.k: each lane forms the partial dot product of its 8 elements (v_dot2_f32_f16, fp32
//     accumulation); the dh/8 partials of the dh/8 rows a lane group holds are combined with a
//     reduce-scatter butterfly, after which every lane owns the complete score of exactly one
//     token: the softmax work (exp2, running max/sum) is done once per token, not per element.
//   * Online softmax state is kept per lane group (the lanes sharing a row) in the log2 domain
//     with a finite "-infinity" so that fully masked tiles need no special case.
#include "hk_internal.h"
#include "elem.h"
#include "attn_ranges.h"

namespace hk {
namespace {


constexpr int kThreads = 256;
constexpr int kWavesPerBlock = 4;
constexpr int kTile = 64;               // tokens per wavefront step
constexpr float kNegBig = -1.0e30f;     // finite stand-in for -inf in running maxima

template <int DT>
__device__ __forceinline__ float dot8(typename Elem<DT>::V8 a, typename Elem<DT>::V8 b)
{
    typedef typename Elem<DT>::V2 half2_t;
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        half2_t x = {a[2 * j], a[2 * j + 1]};
        half2_t y = {b[2 * j], b[2 * j + 1]};
        s = Elem<DT>::dot2(x, y, s);
    }
    return s;
}

using ranges::range_begin;

template <int DH, int DT>
__global__ __launch_bounds__(kThreads) void flash_decode_kernel(
    const typename Elem<DT>::T *__restrict__ q,
    const typename Elem<DT>::T *__restrict__ K0, const typename Elem<DT>::T *__restrict__ V0,
    const typename Elem<DT>::T *__restrict__ K1, const typename Elem<DT>::T *__restrict__ V1,
    int L0, int L1, int64_t total, int W, float scale_log2e,
    float *__restrict__ partial)
{
    typedef typename Elem<DT>::T elem_t;
    typedef typename Elem<DT>::V8 half8_t;
    constexpr int LPR = DH / 8;          // lanes per row
    constexpr int RPL = 64 / LPR;        // rows per load instruction == lane groups per wavefront
    constexpr int NL = LPR;              // loads per lane per 64-token tile

    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6));   // wavefront-uniform
    if (w >= W) return;                  // whole wavefronts leave; the kernel has no barrier
    const int g = lane / LPR, c = lane % LPR;
    const int L = L0 + L1;

    int64_t p = range_begin(w, total, W);
    const int64_t p_end = range_begin(w + 1, total, W);
    while (p < p_end) {
        const int bh = (int)(p / L);
        const int t_first = (int)(p - (int64_t)bh * L);
        const int64_t pair_end = (int64_t)(bh + 1) * L;
        const int t_last = (int)((p_end < pair_end ? p_end : pair_end) - (int64_t)bh * L);   // tokens [t_first, t_last) of pair bh

        const half8_t qv = *reinterpret_cast<const half8_t *>(q + (int64_t)bh * DH + c * 8);
        float m_run = kNegBig, l_run = 0.f;
        float acc[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = 0.f;

        // the part of [t_first, t_last) inside the first segment, then the part inside the second
#pragma unroll 1
        for (int seg = 0; seg < 2; ++seg) {
            const int s_lo = seg ? L0 : 0, s_hi = seg ? L : L0;
            const int a = t_first > s_lo ? t_first : s_lo, b = t_last < s_hi ? t_last : s_hi;
            if (a >= b) continue;
            const int Ls = seg ? L1 : L0;
            const elem_t *Kp = (seg ? K1 : K0) + (int64_t)bh * Ls * DH;
            const elem_t *Vp = (seg ? V1 : V0) + (int64_t)bh * Ls * DH;
            const int t_begin = a - s_lo, t_end = b - s_lo;        // token range inside the segment

            for (int tb = t_begin; tb < t_end; tb += kTile) {
                half8_t kr[NL], vr[NL];
#pragma unroll
                for (int i = 0; i < NL; ++i) {
                    int t = tb + i * RPL + g;
                    if (t >= t_end) t = t_end - 1;                 // clamp; the score is masked below
                    kr[i] = __builtin_nontemporal_load(reinterpret_cast<const half8_t *>(Kp + (int64_t)t * DH + c * 8));
                }
#pragma unroll
                for (int i = 0; i < NL; ++i) {
                    int t = tb + i * RPL + g;
                    if (t >= t_end) t = t_end - 1;
                    vr[i] = __builtin_nontemporal_load(reinterpret_cast<const half8_t *>(Vp + (int64_t)t * DH + c * 8));
                }

                // partial dot products, then reduce-scatter over the LPR lanes of a group
                float pd[NL];
#pragma unroll
                for (int i = 0; i < NL; ++i) pd[i] = dot8<DT>(qv, kr[i]);
#pragma unroll
                for (int h = NL / 2; h >= 1; h >>= 1) {
                    const bool up = (c & h) != 0;
#pragma unroll
                    for (int i = 0; i < h; ++i) {
                        const float send = up ? pd[i] : pd[i + h];
                        const float keep = up ? pd[i + h] : pd[i];
                        pd[i] = keep + __shfl_xor(send, h, 64);
                    }
                }
                // lane (g, c) now owns the score of token tb + c*RPL + g
                const int my_t = tb + c * RPL + g;
                const float s = (my_t < t_end) ? pd[0] * scale_log2e : -INFINITY;

                float m_tile = s;
#pragma unroll
                for (int h = LPR / 2; h >= 1; h >>= 1) m_tile = fmaxf(m_tile, __shfl_xor(m_tile, h, 64));
                const float m_new = fmaxf(m_run, m_tile);
                const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
                const float pe = __builtin_amdgcn_exp2f(s - m_new);
                m_run = m_new;
                l_run = l_run * alpha + pe;
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[j] *= alpha;

#pragma unroll
                for (int i = 0; i < NL; ++i) {
                    const float wgt = __shfl(pe, g * LPR + i, 64);   // weight of token tb + i*RPL + g
#pragma unroll
                    for (int j = 0; j < 8; ++j) acc[j] = __builtin_fmaf(wgt, (float)vr[i][j], acc[j]);
                }
            }
        }

        // ---- combine the lane groups of the wavefront: l over the lanes of a group, then (m, l, o) over groups
#pragma unroll
        for (int h = LPR / 2; h >= 1; h >>= 1) l_run += __shfl_xor(l_run, h, 64);
#pragma unroll
        for (int off = LPR; off < 64; off <<= 1) {
            const float m_o = __shfl_xor(m_run, off, 64);
            const float l_o = __shfl_xor(l_run, off, 64);
            const float m_new = fmaxf(m_run, m_o);
            const float sa = __builtin_amdgcn_exp2f(m_run - m_new), sb = __builtin_amdgcn_exp2f(m_o - m_new);
            l_run = l_run * sa + l_o * sb;
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] = acc[j] * sa + __shfl_xor(acc[j], off, 64) * sb;
            m_run = m_new;
        }
        if (g == 0) {
            float *dst = partial + ((int64_t)w + bh) * (DH + 2);
#pragma unroll
            for (int j = 0; j < 8; ++j) dst[2 + c * 8 + j] = acc[j];
            if (c == 0) { dst[0] = m_run; dst[1] = l_run; }
        }
        p = (int64_t)bh * L + t_last;
    }
}

// Log-sum-exp merge of the partials of one (sequence, head): those of the wavefronts whose range
// meets the pair's positions [bh L, (bh+1) L), at indices (wavefront + bh).
template <int DH, int DT>
__global__ __launch_bounds__(DH) void merge_partials_kernel(const float *__restrict__ partial, int L, int64_t total,
                                                            int W, typename Elem<DT>::T *__restrict__ out, float2 *__restrict__ lse)
{
    const int bh = blockIdx.x, e = threadIdx.x;
    const int64_t lo = (int64_t)bh * L, hi = lo + L - 1;       // first and last position of the pair
    const int w_first = ranges::owner(lo, total, W), w_last = ranges::owner(hi, total, W);
    const float *src = partial + ((int64_t)w_first + bh) * (DH + 2);
    const int n = w_last - w_first + 1;
    float mx = kNegBig;
    for (int i = 0; i < n; ++i) mx = fmaxf(mx, src[i * (DH + 2)]);
    float o = 0.f, l = 0.f;
    for (int i = 0; i < n; ++i) {
        const float wgt = __builtin_amdgcn_exp2f(src[i * (DH + 2)] - mx);
        o = __builtin_fmaf(wgt, src[i * (DH + 2) + 2 + e], o);
        l = __builtin_fmaf(wgt, src[i * (DH + 2) + 1], l);
    }
    out[(int64_t)bh * DH + e] = (typename Elem<DT>::T)(o / l);
    if (lse && e == 0) lse[bh] = make_float2(mx, l);
}

template <int DH, int DT>
hipError_t launch_dh(const AttnArgs &a, hipStream_t s)
{
    typedef typename Elem<DT>::T elem_t;
    const int L = a.L0 + a.L1;
    const int64_t total = (int64_t)a.BH * L;
    const float scale_log2e = a.scale * 1.4426950408889634f;
    const unsigned blocks = (unsigned)((a.n_waves + kWavesPerBlock - 1) / kWavesPerBlock);
    hipLaunchKernelGGL((flash_decode_kernel<DH, DT>), dim3(blocks), dim3(kThreads), 0, s,
                       static_cast<const elem_t *>(a.q),
                       static_cast<const elem_t *>(a.K0), static_cast<const elem_t *>(a.V0),
                       static_cast<const elem_t *>(a.K1), static_cast<const elem_t *>(a.V1),
                       a.L0, a.L1, total, a.n_waves, scale_log2e, a.partial);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && a.after_main) e = hipEventRecord(a.after_main, s);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((merge_partials_kernel<DH, DT>), dim3((unsigned)a.BH), dim3(DH), 0, s,
                       a.partial, L, total, a.n_waves, static_cast<elem_t *>(a.out), a.lse);
    return hipGetLastError();
}

// out = (w_a out_a + w_b out_b) / (w_a + w_b), w_x = l_x 2^(m_x - max(m_a, m_b)): the log-sum-exp join of two token
// segments.  A segment without tokens has denominator 0 and drops out.  4 elements per thread.
template <int DT>
__global__ __launch_bounds__(256) void segment_join_kernel(const typename Elem<DT>::T *__restrict__ out_a, const float2 *__restrict__ lse_a,
                                                           const typename Elem<DT>::T *__restrict__ out_b, const float2 *__restrict__ lse_b,
                                                           typename Elem<DT>::T *__restrict__ out, int64_t n4, int dh4)
{
    typedef typename Elem<DT>::T elem_t;
    typedef elem_t half4_t __attribute__((ext_vector_type(4)));
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= n4) return;
    const int64_t bh = idx / dh4;
    const float2 sa = lse_a[bh], sb = lse_b[bh];
    const float m = fmaxf(sa.x, sb.x);
    const float wa = sa.y * __builtin_amdgcn_exp2f(sa.x - m), wb = sb.y * __builtin_amdgcn_exp2f(sb.x - m);
    const half4_t a = reinterpret_cast<const half4_t *>(out_a)[idx], b = reinterpret_cast<const half4_t *>(out_b)[idx];
    const float inv = wa + wb > 0.f ? 1.0f / (wa + wb) : 0.f;
    half4_t o;
#pragma unroll
    for (int j = 0; j < 4; ++j) o[j] = (elem_t)((wa * (float)a[j] + wb * (float)b[j]) * inv);
    reinterpret_cast<half4_t *>(out)[idx] = o;
}

}  // namespace

hipError_t launch_segment_join(const void *out_a, const float2 *lse_a, const void *out_b, const float2 *lse_b, void *out,
                               int BH, int head_dim, int dtype, hipStream_t s)
{
    if (BH <= 0) return hipSuccess;
    if (head_dim % 4 != 0) return hipErrorInvalidValue;
    const int64_t n4 = (int64_t)BH * (head_dim / 4);
    const unsigned blocks = (unsigned)((n4 + 255) / 256);
    if (dtype == 1)
        hipLaunchKernelGGL(segment_join_kernel<1>, dim3(blocks), dim3(256), 0, s, static_cast<const __bf16 *>(out_a), lse_a,
                           static_cast<const __bf16 *>(out_b), lse_b, static_cast<__bf16 *>(out), n4, head_dim / 4);
    else
        hipLaunchKernelGGL(segment_join_kernel<0>, dim3(blocks), dim3(256), 0, s, static_cast<const _Float16 *>(out_a), lse_a,
                           static_cast<const _Float16 *>(out_b), lse_b, static_cast<_Float16 *>(out), n4, head_dim / 4);
    return hipGetLastError();
}

int attn_wavefronts(int64_t BH, int64_t L, int splits, int resident)
{
    const int64_t total = BH * L;
    if (total <= 0) return 0;
    int64_t W;
    if (splits > 0) {
        W = BH * splits;                                       // `splits` equal token ranges per pair
    } else {
        W = resident;                                          // every wavefront resident: one round
        const int64_t by_work = (total + 2 * kTile - 1) / (2 * kTile);   // at least ~128 tokens each
        if (W > by_work) W = by_work;
    }
    if (W > total) W = total;                                  // no empty range
    if (W > kAttnMaxWaves) W = kAttnMaxWaves;
    return (int)W;
}

hipError_t launch_flash_decode(const AttnArgs &a, hipStream_t s)
{
    if (a.BH <= 0) return hipSuccess;
    if (a.n_waves <= 0 || a.n_waves > kAttnMaxWaves || (int64_t)a.n_waves > (int64_t)a.BH * (a.L0 + a.L1))
        return hipErrorInvalidValue;
    if (a.head_dim == 128) return a.dtype == 1 ? launch_dh<128, 1>(a, s) : launch_dh<128, 0>(a, s);
    if (a.head_dim == 64) return a.dtype == 1 ? launch_dh<64, 1>(a, s) : launch_dh<64, 0>(a, s);
    return hipErrorInvalidValue;
}

}  // namespace hk
