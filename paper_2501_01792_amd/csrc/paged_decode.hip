// Single-query attention over a paged hybrid cache (Sec. 4.1, 4.2.1): every request's context is a
// list of logical blocks of `block_tokens` tokens, each either a KV block (its K/V rows sit in the KV
// pool) or an ACT block (its checkpoints sit in the activation pool; its K/V rows have just been
// regenerated into a pool of the same shape as the KV pool).  A per-request block table maps logical
// block -> (kind, physical block number).  Requests have their own lengths.  This is the role of the
// paper's attention kernel that reads both kinds of buffer (Sec. 5.1).
//
// Same organisation as the contiguous kernel (flash_decode.hip): the token positions of all
// (request, head) pairs form one line, pair-major, of H * sum(len) positions; it is cut into W equal
// ranges, one per resident wavefront; a wavefront emits one partial per pair it touches at index
// (wavefront + pair); a second kernel merges each pair's run of partials.  What differs is the address
// of a token: the block table is read with scalar loads (one entry per load instruction's group of
// rows, which never straddles a block), and tiles are aligned to 64 tokens inside a pair so that the
// rows of one load instruction share a block.
#include "hk_internal.h"
#include "elem.h"
#include "attn_ranges.h"

namespace hk {
namespace {

constexpr int kThreads = 256;
constexpr int kWavesPerBlock = 4;
constexpr int kTile = 64;
constexpr float kNegBig = -1.0e30f;

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

using ranges::effective_waves;
using ranges::range_begin;

// Request that holds position p of the pair-major line: the last r with H * cu[r] <= p (cu has B + 1 entries).
__device__ __forceinline__ int request_of(const int64_t *__restrict__ cu, int B, int H, int64_t p)
{
    int lo = 0, hi = B;                  // invariant: H cu[lo] <= p < H cu[hi]
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if ((int64_t)H * cu[mid] <= p) lo = mid; else hi = mid;
    }
    return lo;
}

template <int DH, int DT>
__global__ __launch_bounds__(kThreads) void paged_decode_kernel(
    const typename Elem<DT>::T *__restrict__ q,
    const typename Elem<DT>::T *__restrict__ K_pool, const typename Elem<DT>::T *__restrict__ V_pool,      // KV blocks
    const typename Elem<DT>::T *__restrict__ K_regen, const typename Elem<DT>::T *__restrict__ V_regen,    // regenerated ACT blocks
    const int32_t *__restrict__ table, int max_blocks, int P_kv, int P_act,
    const int32_t *__restrict__ seq_len, const int64_t *__restrict__ cu,
    int B, int H, int blk_log2, int64_t total_host, const int64_t *__restrict__ total_dev, int W, float scale_log2e,
    float *__restrict__ partial)
{
    typedef typename Elem<DT>::V8 half8_t;
    constexpr int LPR = DH / 8, RPL = 64 / LPR, NL = LPR;
    // positions of the line: known to the host, or (tables built on the device) H * total_dev[0] <= the host's bound
    const int64_t total = total_dev ? (int64_t)H * total_dev[0] : total_host;
    // The launch may be sized for more positions than the device finds (an upper bound on the host): then only
    // the first `total` wavefronts work, so that no range between two working wavefronts is empty and every
    // partial slot the merge reads has been written.  The merge derives the same number.
    W = effective_waves(W, total);

    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6));
    if (w >= W) return;                  // whole wavefronts leave; the kernel has no barrier
    const int g = lane / LPR, c = lane % LPR;
    const int blk = 1 << blk_log2;
    const int64_t blk_elems = (int64_t)H * blk * DH;       // elements of one pool block

    int64_t p = range_begin(w, total, W);
    const int64_t p_end = range_begin(w + 1, total, W);
    int r = request_of(cu, B, H, p);
    while (p < p_end) {
        // position p -> (request r, head h, token t_first); requests without tokens are stepped over
        int64_t base = (int64_t)H * cu[r];
        int len = seq_len[r];
        while (p >= base + (int64_t)H * len) { ++r; base = (int64_t)H * cu[r]; len = seq_len[r]; }
        const int h = (int)((p - base) / len);
        const int t_first = (int)(p - base - (int64_t)h * len);
        const int64_t pair_end = base + (int64_t)(h + 1) * len;
        const int t_last = (int)((p_end < pair_end ? p_end : pair_end) - (base + (int64_t)h * len));   // tokens [t_first, t_last)
        const int pair = r * H + h;
        const int32_t *tab = table + (int64_t)r * max_blocks;
        const int last_block = (t_last - 1) >> blk_log2;

        const half8_t qv = *reinterpret_cast<const half8_t *>(q + (int64_t)pair * DH + c * 8);
        float m_run = kNegBig, l_run = 0.f;
        float acc[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = 0.f;

        for (int tb = t_first & ~(kTile - 1); tb < t_last; tb += kTile) {
            half8_t kr[NL], vr[NL];
            // Address of the rows of load group i: a wavefront-uniform block base (scalar registers) plus a
            // 32-bit lane offset.  A 64-token tile meets at most four blocks (block_tokens >= 16); rows
            // tb + i RPL .. + RPL - 1 lie in one of them (block_tokens is a multiple of RPL).  Groups past the
            // last token are redirected to the last token's block and row, and masked below.
            int64_t kv_base[4];          // element offset of (block, head h, token 0 of the pair) in its pool
            bool kv_act[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                int bi = (tb >> blk_log2) + j;
                bi = bi < last_block ? bi : last_block;
                const int32_t e = __builtin_amdgcn_readfirstlane(tab[bi]);
                bool is_act = e < 0;
                int pb = is_act ? ~e : e;
                if ((is_act ? P_act : P_kv) <= 0) { is_act = !is_act; pb = 0; }   // a corrupt table cannot leave
                const int P = is_act ? P_act : P_kv;                              // the pools (one is not empty)
                pb = pb < P ? pb : P - 1;
                kv_act[j] = is_act;
                kv_base[j] = (int64_t)pb * blk_elems + (int64_t)h * (blk * DH) - (int64_t)(bi << blk_log2) * DH;   // + t * DH
            }
            auto lane_off = [&](int i) {
                int t = tb + i * RPL + g;
                t = t < t_last ? t : t_last - 1;
                return (uint32_t)(t * DH + c * 8);
            };
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                const int j = (i * RPL) >> blk_log2;               // 0..3, wavefront-uniform
                const int64_t b = j == 0 ? kv_base[0] : j == 1 ? kv_base[1] : j == 2 ? kv_base[2] : kv_base[3];
                const bool a = j == 0 ? kv_act[0] : j == 1 ? kv_act[1] : j == 2 ? kv_act[2] : kv_act[3];
                kr[i] = __builtin_nontemporal_load(reinterpret_cast<const half8_t *>((a ? K_regen : K_pool) + b + lane_off(i)));
            }
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                const int j = (i * RPL) >> blk_log2;
                const int64_t b = j == 0 ? kv_base[0] : j == 1 ? kv_base[1] : j == 2 ? kv_base[2] : kv_base[3];
                const bool a = j == 0 ? kv_act[0] : j == 1 ? kv_act[1] : j == 2 ? kv_act[2] : kv_act[3];
                vr[i] = __builtin_nontemporal_load(reinterpret_cast<const half8_t *>((a ? V_regen : V_pool) + b + lane_off(i)));
            }

            float pd[NL];
#pragma unroll
            for (int i = 0; i < NL; ++i) pd[i] = dot8<DT>(qv, kr[i]);
#pragma unroll
            for (int hh = NL / 2; hh >= 1; hh >>= 1) {
                const bool up = (c & hh) != 0;
#pragma unroll
                for (int i = 0; i < hh; ++i) {
                    const float send = up ? pd[i] : pd[i + hh];
                    const float keep = up ? pd[i + hh] : pd[i];
                    pd[i] = keep + __shfl_xor(send, hh, 64);
                }
            }
            // lane (g, c) now owns the score of token tb + c*RPL + g
            const int my_t = tb + c * RPL + g;
            const float s = (my_t >= t_first && my_t < t_last) ? pd[0] * scale_log2e : -INFINITY;

            float m_tile = s;
#pragma unroll
            for (int hh = LPR / 2; hh >= 1; hh >>= 1) m_tile = fmaxf(m_tile, __shfl_xor(m_tile, hh, 64));
            const float m_new = fmaxf(m_run, m_tile);
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
            const float pe = __builtin_amdgcn_exp2f(s - m_new);
            m_run = m_new;
            l_run = l_run * alpha + pe;
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] *= alpha;
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                const float wgt = __shfl(pe, g * LPR + i, 64);
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[j] = __builtin_fmaf(wgt, (float)vr[i][j], acc[j]);
            }
        }

#pragma unroll
        for (int hh = LPR / 2; hh >= 1; hh >>= 1) l_run += __shfl_xor(l_run, hh, 64);
#pragma unroll
        for (int o2 = LPR; o2 < 64; o2 <<= 1) {
            const float m_o = __shfl_xor(m_run, o2, 64);
            const float l_o = __shfl_xor(l_run, o2, 64);
            const float m_new = fmaxf(m_run, m_o);
            const float sa = __builtin_amdgcn_exp2f(m_run - m_new), sb = __builtin_amdgcn_exp2f(m_o - m_new);
            l_run = l_run * sa + l_o * sb;
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] = acc[j] * sa + __shfl_xor(acc[j], o2, 64) * sb;
            m_run = m_new;
        }
        if (g == 0) {
            float *dst = partial + ((int64_t)w + pair) * (DH + 2);
#pragma unroll
            for (int j = 0; j < 8; ++j) dst[2 + c * 8 + j] = acc[j];
            if (c == 0) { dst[0] = m_run; dst[1] = l_run; }
        }
        p = base + (int64_t)h * len + t_last;
    }
}

// Merge of the partials of one (request, head): positions [H cu[r] + h len, + len) of the line.
template <int DH, int DT>
__global__ __launch_bounds__(DH) void paged_merge_kernel(const float *__restrict__ partial,
                                                         const int32_t *__restrict__ seq_len, const int64_t *__restrict__ cu,
                                                         int H, int64_t total_host, const int64_t *__restrict__ total_dev, int W,
                                                         typename Elem<DT>::T *__restrict__ out, float2 *__restrict__ lse)
{
    const int64_t total = total_dev ? (int64_t)H * total_dev[0] : total_host;   // > 0 whenever a pair has tokens
    W = effective_waves(W, total);       // as in the streaming kernel: no empty range among the working wavefronts
    const int pair = blockIdx.x, e = threadIdx.x;
    const int r = pair / H, h = pair % H;
    const int len = seq_len[r];
    if (len <= 0 || total <= 0) {        // no context: the softmax is over nothing; define the output as zero
        out[(int64_t)pair * DH + e] = (typename Elem<DT>::T)0.f;
        if (lse && e == 0) lse[pair] = make_float2(kNegBig, 0.f);
        return;
    }
    const int64_t lo = (int64_t)H * cu[r] + (int64_t)h * len, hi = lo + len - 1;
    const int w_first = ranges::owner(lo, total, W), w_last = ranges::owner(hi, total, W);
    const float *src = partial + ((int64_t)w_first + pair) * (DH + 2);
    const int n = w_last - w_first + 1;
    float mx = kNegBig;
    for (int i = 0; i < n; ++i) mx = fmaxf(mx, src[i * (DH + 2)]);
    float o = 0.f, l = 0.f;
    for (int i = 0; i < n; ++i) {
        const float wgt = __builtin_amdgcn_exp2f(src[i * (DH + 2)] - mx);
        o = __builtin_fmaf(wgt, src[i * (DH + 2) + 2 + e], o);
        l = __builtin_fmaf(wgt, src[i * (DH + 2) + 1], l);
    }
    out[(int64_t)pair * DH + e] = (typename Elem<DT>::T)(o / l);
    if (lse && e == 0) lse[pair] = make_float2(mx, l);
}

template <int DH, int DT>
hipError_t launch_dh(const PagedAttnArgs &a, hipStream_t s)
{
    typedef typename Elem<DT>::T elem_t;
    const int64_t total = (int64_t)a.H * a.total_tokens;
    const float scale_log2e = a.scale * 1.4426950408889634f;
    int blk_log2 = 0;
    while ((1 << blk_log2) < a.block_tokens) ++blk_log2;
    if (total > 0) {
        const unsigned blocks = (unsigned)((a.n_waves + kWavesPerBlock - 1) / kWavesPerBlock);
        hipLaunchKernelGGL((paged_decode_kernel<DH, DT>), dim3(blocks), dim3(kThreads), 0, s,
                           static_cast<const elem_t *>(a.q),
                           static_cast<const elem_t *>(a.K_pool), static_cast<const elem_t *>(a.V_pool),
                           static_cast<const elem_t *>(a.K_regen), static_cast<const elem_t *>(a.V_regen),
                           a.block_table, a.max_blocks, a.P_kv, a.P_act, a.seq_len, a.cu_tokens,
                           a.B, a.H, blk_log2, total, a.total_dev, a.n_waves, scale_log2e, a.partial);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((paged_merge_kernel<DH, DT>), dim3((unsigned)(a.B * a.H)), dim3(DH), 0, s,
                       a.partial, a.seq_len, a.cu_tokens, a.H, total > 0 ? total : 1, a.total_dev, a.n_waves > 0 ? a.n_waves : 1,
                       static_cast<elem_t *>(a.out), a.lse);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_paged_decode(const PagedAttnArgs &a, hipStream_t s)
{
    if (a.B <= 0) return hipSuccess;
    if (a.block_tokens < 16 || (a.block_tokens & (a.block_tokens - 1)) != 0) return hipErrorInvalidValue;
    if (a.total_tokens > 0 && (a.n_waves <= 0 || (int64_t)a.n_waves > (int64_t)a.H * a.total_tokens)) return hipErrorInvalidValue;
    if (a.head_dim == 128) return a.dtype == 1 ? launch_dh<128, 1>(a, s) : launch_dh<128, 0>(a, s);
    if (a.head_dim == 64) return a.dtype == 1 ? launch_dh<64, 1>(a, s) : launch_dh<64, 0>(a, s);
    return hipErrorInvalidValue;
}

}  // namespace hk
