// Single-query attention (Eq. 4) over cached ++ regenerated K/V (Eq. 3) for gfx950.
//
// The decode query of each (sequence, head) attends over every context token.  With one query
// per head the work is one pass over K and one over V: ~1 FLOP per byte, so the kernel is an HBM
// streaming kernel and is organised around the loads, not the arithmetic:
//   * The context of a (sequence, head) is two contiguous token segments (the cached rows and
//     the regenerated rows); they are never copied together.  The token axis of each segment is
//     cut into chunks; one workgroup per (sequence*head, chunk).  Every workgroup (4 wavefronts) streams one
//     chunk and emits an un-normalised partial (m, l, o[dh]); a second tiny kernel merges the
//     partials of a (sequence, head) by log-sum-exp.  With a single chunk the workgroup writes
//     the final output itself.
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

namespace hk {
namespace {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

constexpr int kThreads = 256;
constexpr int kWaves = 4;
constexpr int kTile = 64;               // tokens per wavefront step
constexpr float kNegBig = -1.0e30f;     // finite stand-in for -inf in running maxima

__device__ __forceinline__ float dot8(half8_t a, half8_t b)
{
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        half2_t x = {a[2 * j], a[2 * j + 1]};
        half2_t y = {b[2 * j], b[2 * j + 1]};
        s = __builtin_amdgcn_fdot2(x, y, s, false);
    }
    return s;
}

template <int DH>
__global__ __launch_bounds__(kThreads) void flash_decode_kernel(
    const _Float16 *__restrict__ q,
    const _Float16 *__restrict__ K0, const _Float16 *__restrict__ V0,
    const _Float16 *__restrict__ K1, const _Float16 *__restrict__ V1,
    int L0, int L1, int chunk, int chunks0, int total_chunks, float scale_log2e,
    float *__restrict__ partial, _Float16 *__restrict__ out)
{
    constexpr int LPR = DH / 8;          // lanes per row
    constexpr int RPL = 64 / LPR;        // rows per load instruction == lane groups per wavefront
    constexpr int NL = LPR;              // loads per lane per 64-token tile
    constexpr int NSTATE = kWaves * RPL; // partial softmax states per workgroup

    __shared__ float s_m[NSTATE];
    __shared__ float s_l[NSTATE];
    __shared__ float s_o[NSTATE][DH];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane / LPR, c = lane % LPR;
    // Workgroups are numbered so that the launch walks the (sequence, head) pairs from the last to the
    // first and, within a pair, the second (regenerated) segment before the first: the rows that the
    // projection kernel wrote most recently are read first, while they are still in the last-level cache.
    const int rev = gridDim.x - 1 - blockIdx.x;
    const int bh = rev / total_chunks;
    const int ck = rev % total_chunks;

    // which segment, which token range
    const bool second = ck >= chunks0;
    const int L = second ? L1 : L0;
    const _Float16 *Kp = (second ? K1 : K0) + (int64_t)bh * L * DH;
    const _Float16 *Vp = (second ? V1 : V0) + (int64_t)bh * L * DH;
    const int t_begin = (second ? ck - chunks0 : ck) * chunk;
    const int t_end = (t_begin + chunk < L) ? t_begin + chunk : L;   // t_begin < L by construction

    const half8_t qv = *reinterpret_cast<const half8_t *>(q + (int64_t)bh * DH + c * 8);

    float m_run = kNegBig, l_run = 0.f;
    float acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = 0.f;

    for (int tb = t_begin + wave * kTile; tb < t_end; tb += kWaves * kTile) {
        half8_t kr[NL], vr[NL];
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            int t = tb + i * RPL + g;
            if (t >= t_end) t = t_end - 1;                 // clamp; the score is masked below
            kr[i] = *reinterpret_cast<const half8_t *>(Kp + (int64_t)t * DH + c * 8);
        }
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            int t = tb + i * RPL + g;
            if (t >= t_end) t = t_end - 1;
            vr[i] = *reinterpret_cast<const half8_t *>(Vp + (int64_t)t * DH + c * 8);
        }

        // partial dot products, then reduce-scatter over the LPR lanes of a group
        float p[NL];
#pragma unroll
        for (int i = 0; i < NL; ++i) p[i] = dot8(qv, kr[i]);
#pragma unroll
        for (int h = NL / 2; h >= 1; h >>= 1) {
            const bool up = (c & h) != 0;
#pragma unroll
            for (int i = 0; i < h; ++i) {
                const float send = up ? p[i] : p[i + h];
                const float keep = up ? p[i + h] : p[i];
                p[i] = keep + __shfl_xor(send, h, 64);
            }
        }
        // lane (g, c) now owns the score of token tb + c*RPL + g
        const int my_t = tb + c * RPL + g;
        float s = (my_t < t_end) ? p[0] * scale_log2e : -INFINITY;

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
            const float w = __shfl(pe, g * LPR + i, 64);   // weight of token tb + i*RPL + g
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] = __builtin_fmaf(w, (float)vr[i][j], acc[j]);
        }
    }

    // ---- combine the lane groups and wavefronts of the workgroup
#pragma unroll
    for (int h = LPR / 2; h >= 1; h >>= 1) l_run += __shfl_xor(l_run, h, 64);
    const int st = wave * RPL + g;
    if (c == 0) { s_m[st] = m_run; s_l[st] = l_run; }
#pragma unroll
    for (int j = 0; j < 8; ++j) s_o[st][c * 8 + j] = acc[j];
    __syncthreads();

    if (tid < DH) {
        float mx = kNegBig;
#pragma unroll
        for (int i = 0; i < NSTATE; ++i) mx = fmaxf(mx, s_m[i]);
        float o = 0.f, l = 0.f;
#pragma unroll
        for (int i = 0; i < NSTATE; ++i) {
            const float w = __builtin_amdgcn_exp2f(s_m[i] - mx);
            o = __builtin_fmaf(w, s_o[i][tid], o);
            l = __builtin_fmaf(w, s_l[i], l);
        }
        if (total_chunks == 1) {
            out[(int64_t)bh * DH + tid] = (_Float16)(o / l);
        } else {
            float *dst = partial + ((int64_t)bh * total_chunks + ck) * (DH + 2);
            dst[2 + tid] = o;
            if (tid == 0) { dst[0] = mx; dst[1] = l; }
        }
    }
}

// Log-sum-exp merge of the per-chunk partials of one (sequence, head).
template <int DH>
__global__ __launch_bounds__(DH) void merge_partials_kernel(const float *__restrict__ partial,
                                                            int total_chunks, _Float16 *__restrict__ out)
{
    const int bh = blockIdx.x, e = threadIdx.x;
    const float *src = partial + (int64_t)bh * total_chunks * (DH + 2);
    float mx = kNegBig;
    for (int i = 0; i < total_chunks; ++i) mx = fmaxf(mx, src[i * (DH + 2)]);
    float o = 0.f, l = 0.f;
    for (int i = 0; i < total_chunks; ++i) {
        const float w = __builtin_amdgcn_exp2f(src[i * (DH + 2)] - mx);
        o = __builtin_fmaf(w, src[i * (DH + 2) + 2 + e], o);
        l = __builtin_fmaf(w, src[i * (DH + 2) + 1], l);
    }
    out[(int64_t)bh * DH + e] = (_Float16)(o / l);
}

template <int DH>
hipError_t launch_dh(const AttnArgs &a, hipStream_t s)
{
    const int chunks0 = (a.L0 + a.chunk - 1) / a.chunk;
    const int total = attn_total_chunks(a.L0, a.L1, a.chunk);
    const float scale_log2e = a.scale * 1.4426950408889634f;
    hipLaunchKernelGGL(flash_decode_kernel<DH>, dim3((unsigned)((int64_t)a.BH * total)), dim3(kThreads), 0, s,
                       static_cast<const _Float16 *>(a.q),
                       static_cast<const _Float16 *>(a.K0), static_cast<const _Float16 *>(a.V0),
                       static_cast<const _Float16 *>(a.K1), static_cast<const _Float16 *>(a.V1),
                       a.L0, a.L1, a.chunk, chunks0, total, scale_log2e,
                       a.partial, static_cast<_Float16 *>(a.out));
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && a.after_main) e = hipEventRecord(a.after_main, s);
    if (e != hipSuccess || total == 1) return e;
    hipLaunchKernelGGL(merge_partials_kernel<DH>, dim3((unsigned)a.BH), dim3(DH), 0, s,
                       a.partial, total, static_cast<_Float16 *>(a.out));
    return hipGetLastError();
}

}  // namespace

int attn_total_chunks(int L0, int L1, int chunk)
{
    return (L0 + chunk - 1) / chunk + (L1 + chunk - 1) / chunk;
}

hipError_t launch_flash_decode(const AttnArgs &a, hipStream_t s)
{
    if (a.BH <= 0) return hipSuccess;
    if ((int64_t)a.BH * attn_total_chunks(a.L0, a.L1, a.chunk) > 0x7fffffffLL) return hipErrorInvalidValue;
    if (a.head_dim == 128) return launch_dh<128>(a, s);
    if (a.head_dim == 64) return launch_dh<64>(a, s);
    return hipErrorInvalidValue;
}

}  // namespace hk
