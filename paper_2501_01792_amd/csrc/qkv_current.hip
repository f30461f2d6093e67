// QKV generation for the current input token of every sequence (Sec. 4.2.2: "QKV generation" of the
// decode step, Eq. 2 with the layer's pre-attention LayerNorm in front), and the write-back of that
// token into one of the two stores: its K/V row into the KV cache, or its layer input into the
// activation checkpoints.
//
//   xhat = LayerNorm(x_cur)                      [B, d]
//   q    = xhat Wq^T + bq                        -> q_out [B, H, dh]
//   k, v = xhat [Wk; Wv]^T + [bk; bv]            -> K_dst, V_dst [B, H, L_cap, dh] at token tok_pos
//
// With B rows only, this is a skinny GEMM whose cost is one pass over the weights (2 d^2 or 6 d^2
// bytes): an HBM streaming kernel.  Three kernels:
//   ln_rows:    one wavefront per row: statistics from a register copy of the row, then the normalised
//               row in fp16 to scratch (and the raw row to the checkpoint store when asked).
//   qkv_block:  one workgroup per (block of 128 output features, part of the reduction axis): its 4
//               wavefronts stream 32 weight rows each from HBM (whole-line loads, several steps in
//               flight, through a private LDS block into MFMA operand layout) and share the matching
//               tile of xhat through LDS, so that xhat is read from L2 once per 128 weight rows
//               (skinny::block_product).  The reduction axis is cut over workgroups only as far as it
//               takes to fill the chip; every part leaves an fp32 partial result in scratch.
//   qkv_finish: sums the parts, adds the bias, rounds to fp16 and scatters to q / K / V.
#include "hk_internal.h"
#include "elem.h"
#include "skinny_mma.h"

namespace hk {
namespace {

using skinny::float16_t;

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// Where the current token of a request goes in a paged cache (QkvArgs): its table entry and its row in the block,
// or row < 0 when the request has no token, the table has no entry for it, or the caller's mask says that the
// token is not to be stored.
struct PagedDst {
    const int32_t *block_table, *seq_len;      // block_table == nullptr: contiguous stores
    const int32_t *store_mask;                 // optional: zero = the request's token is not stored
    int max_blocks, blk_log2, P_kv, P_act;
};
__device__ __forceinline__ void paged_slot(const PagedDst &p, int b, int32_t &entry, int &row)
{
    row = -1;
    entry = 0;
    if (p.store_mask && p.store_mask[b] == 0) return;
    const int t = p.seq_len[b] - 1;
    if (t < 0) return;
    const int bi = t >> p.blk_log2;
    if (bi >= p.max_blocks) return;
    entry = p.block_table[(int64_t)b * p.max_blocks + bi];
    row = t & ((1 << p.blk_log2) - 1);
}

constexpr int kMaxVec = 5;               // rows of up to 256 * 8 * 5 = 10240 elements are held in registers

// xhat[r, :] = ((x[r, :] - mean) * rstd) * gamma + beta in fp32, rounded once to the storage type.  One workgroup per row; the
// row, gamma and beta are requested together (the launch is short and cold: one memory latency instead of two),
// mean and centred sum of squares come from the register copy.
template <int DT>
__global__ __launch_bounds__(256) void ln_rows_kernel(const typename Elem<DT>::T *__restrict__ x,
                                                      const typename Elem<DT>::T *__restrict__ gamma,
                                                      const typename Elem<DT>::T *__restrict__ beta,
                                                      typename Elem<DT>::T *__restrict__ xhat,
                                                      typename Elem<DT>::T *__restrict__ act_dst, int64_t act_row_stride,
                                                      int d, float eps, PagedDst pd)
{
    typedef typename Elem<DT>::T elem_t;
    typedef typename Elem<DT>::V8 half8_t;
    __shared__ float red[2][4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t row = blockIdx.x;                        // grid = rows
    const half8_t *p = reinterpret_cast<const half8_t *>(x + row * d);
    const half8_t *g8 = reinterpret_cast<const half8_t *>(gamma), *b8 = reinterpret_cast<const half8_t *>(beta);
    const int nvec = d >> 3;                               // <= 256 kMaxVec (checked by the launcher)
    half8_t zero;
#pragma unroll
    for (int j = 0; j < 8; ++j) zero[j] = (elem_t)0.f;
    half8_t v[kMaxVec], g[kMaxVec], be[kMaxVec];
#pragma unroll
    for (int i = 0; i < kMaxVec; ++i) {
        const int idx = tid + 256 * i;
        const bool ok = idx < nvec;
        v[i] = ok ? p[idx] : zero;
        g[i] = ok ? g8[idx] : zero;
        be[i] = ok ? b8[idx] : zero;
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < kMaxVec; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) s += (float)v[i][j];
    s = wave_sum(s);
    if (lane == 0) red[0][wave] = s;
    __syncthreads();
    const float mean = (red[0][0] + red[0][1] + red[0][2] + red[0][3]) / (float)d;
    float sq = 0.f;
#pragma unroll
    for (int i = 0; i < kMaxVec; ++i) {
        if (tid + 256 * i < nvec) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float c = (float)v[i][j] - mean;
                sq = __builtin_fmaf(c, c, sq);
            }
        }
    }
    sq = wave_sum(sq);
    if (lane == 0) red[1][wave] = sq;
    __syncthreads();
    const float rstd = 1.0f / __builtin_sqrtf((red[1][0] + red[1][1] + red[1][2] + red[1][3]) / (float)d + eps);
    half8_t *dst = reinterpret_cast<half8_t *>(xhat + row * d);
    half8_t *ckpt = act_dst ? reinterpret_cast<half8_t *>(act_dst + row * act_row_stride) : nullptr;
    if (pd.block_table) {                                  // paged: the row of the ACT block named by the table, if it is one
        int32_t entry;
        int r;
        paged_slot(pd, (int)row, entry, r);
        ckpt = (act_dst && r >= 0 && entry < 0 && ~entry < pd.P_act)
                   ? reinterpret_cast<half8_t *>(act_dst + ((((int64_t)~entry) << pd.blk_log2) + r) * d) : nullptr;
    }
#pragma unroll
    for (int i = 0; i < kMaxVec; ++i) {
        const int idx = tid + 256 * i;
        if (idx < nvec) {
            half8_t o;
#pragma unroll
            for (int j = 0; j < 8; ++j)
                o[j] = (elem_t)__builtin_fmaf(((float)v[i][j] - mean) * rstd, (float)g[i][j], (float)be[i][j]);
            dst[idx] = o;
            if (ckpt) ckpt[idx] = v[i];
        }
    }
}

// Feature blocks: 128 rows of Wq (ceil(d / 128) blocks), then 128 rows of [Wk; Wv] (ceil(2d / 128) blocks),
// so that a block never straddles the two weight arrays.  Partials: part[ks][m][n], n in [0, 3d) fp32.
template <int RB, int DT>
__global__ __launch_bounds__(256) void qkv_block_kernel(
    const _Float16 *__restrict__ xhat, const _Float16 *__restrict__ Wq, const _Float16 *__restrict__ Wkv,
    float *__restrict__ part, int B, int d, int q_blocks, int steps_per_part)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int blk = blockIdx.x, ks = blockIdx.y;
    const bool is_q = blk < q_blocks;
    const int n0 = is_q ? blk * 128 : (blk - q_blocks) * 128;              // first row inside its weight array
    const int n_rows = (is_q ? d : 2 * d) - n0 < 128 ? (is_q ? d : 2 * d) - n0 : 128;
    const _Float16 *W = (is_q ? Wq : Wkv) + (int64_t)n0 * d;
    const int steps = d / 64;
    const int k_begin = ks * steps_per_part;
    const int k_steps = steps - k_begin < steps_per_part ? steps - k_begin : steps_per_part;
    float16_t acc[RB];
    float m1[4], m2[4];
    _Float16 first[4];
    skinny::block_product<RB, true, false, DT>(W, n_rows, d, xhat, B, d, k_begin, k_steps, smem, acc, m1, m2, first);
    // acc[rb][r]: row (sequence) 32 rb + 8 (r/4) + 4 (lane/32) + r%4, feature 32 wave + lane%32 of the block
    const int ln = lane & 31, lh = lane >> 5;
    const int c = 32 * wave + ln;
    if (c < n_rows) {
        const int n = (is_q ? 0 : d) + n0 + c;
        float *dst = part + (int64_t)ks * B * 3 * d + n;
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = 32 * rb + 8 * (r >> 2) + 4 * lh + (r & 3);
                if (m < B) dst[(int64_t)m * 3 * d] = acc[rb][r];
            }
    }
}

// out[m][n] = sum_ks part[ks][m][n] + bias[n], rounded to the storage type, 4 features per thread, scattered to q / K / V.
template <int DT>
__global__ __launch_bounds__(256) void qkv_finish_kernel(
    const float *__restrict__ part, int parts, const typename Elem<DT>::T *__restrict__ bq,
    const typename Elem<DT>::T *__restrict__ bkv, typename Elem<DT>::T *__restrict__ q_out,
    typename Elem<DT>::T *__restrict__ K_dst, typename Elem<DT>::T *__restrict__ V_dst,
    int B, int d, int n_out, int n_heads, int head_dim, int L_cap, int tok_pos, PagedDst pd)
{
    typedef typename Elem<DT>::T elem_t;
    typedef elem_t half4_t __attribute__((ext_vector_type(4)));
    const int per_row = n_out / 4;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)B * per_row) return;
    const int m = (int)(idx / per_row), n = (int)(idx % per_row) * 4;
    const int64_t stride = (int64_t)B * 3 * d;
    const float *src = part + (int64_t)m * 3 * d + n;
    float4_t sum = *reinterpret_cast<const float4_t *>(src);
    for (int ks = 1; ks < parts; ++ks) sum += *reinterpret_cast<const float4_t *>(src + ks * stride);
    const int which = n / d, nn = n - which * d;                           // 0: q, 1: k, 2: v
    const elem_t *bias = which == 0 ? bq + nn : bkv + (which - 1) * d + nn;
    half4_t o;
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] = (elem_t)(sum[i] + (float)bias[i]);
    if (which == 0) {
        *reinterpret_cast<half4_t *>(q_out + (int64_t)m * d + nn) = o;
    } else {
        const int h = nn / head_dim, e = nn % head_dim;
        elem_t *dst = which == 1 ? K_dst : V_dst;
        if (pd.block_table) {                              // paged: the row of the KV block named by the table, if it is one
            int32_t entry;
            int r;
            paged_slot(pd, m, entry, r);
            if (r >= 0 && entry >= 0 && entry < pd.P_kv)
                *reinterpret_cast<half4_t *>(dst + (((((int64_t)entry * n_heads + h)) << pd.blk_log2) + r) * head_dim + e) = o;
        } else {
            *reinterpret_cast<half4_t *>(dst + (((int64_t)m * n_heads + h) * L_cap + tok_pos) * head_dim + e) = o;
        }
    }
}

PagedDst paged_dst(const QkvArgs &a)
{
    return PagedDst{a.block_table, a.seq_len, a.store_mask, a.max_blocks, a.blk_log2, a.P_kv, a.P_act};
}

template <int DT>
hipError_t launch_ln_rows(const QkvArgs &a, hipStream_t s)
{
    typedef typename Elem<DT>::T elem_t;
    hipLaunchKernelGGL(ln_rows_kernel<DT>, dim3((unsigned)a.B), dim3(256), 0, s,
                       static_cast<const elem_t *>(a.x), static_cast<const elem_t *>(a.ln_w),
                       static_cast<const elem_t *>(a.ln_b), static_cast<elem_t *>(a.xhat),
                       static_cast<elem_t *>(a.act_dst), a.act_row_stride, a.d, a.eps, paged_dst(a));
    return hipGetLastError();
}

// The operands are handed to skinny::block_product as 16-bit elements of either format (same size and addressing).
template <int RB, int DT>
hipError_t launch_block(const QkvArgs &a, int parts, int steps_per_part, hipStream_t s)
{
    const int q_blocks = (a.d + 127) / 128, kv_blocks = a.K_dst ? (2 * a.d + 127) / 128 : 0;
    auto kern = qkv_block_kernel<RB, DT>;
    constexpr int lds = skinny::block_lds_bytes<RB>();
    static LdsOnce lds_once;
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kern), lds, lds_once);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)(q_blocks + kv_blocks), (unsigned)parts), dim3(256), lds, s,
                       static_cast<const _Float16 *>(a.xhat), static_cast<const _Float16 *>(a.Wq),
                       static_cast<const _Float16 *>(a.Wkv), a.part, a.B, a.d, q_blocks, steps_per_part);
    return hipGetLastError();
}

template <int DT>
hipError_t launch_dt(const QkvArgs &a, hipStream_t s)
{
    typedef typename Elem<DT>::T elem_t;
    hipError_t e = launch_ln_rows<DT>(a, s);
    if (e != hipSuccess) return e;
    int parts, steps_per_part;
    qkv_parts(a.d, &parts, &steps_per_part);
    if ((size_t)parts * a.B * 3 * a.d > a.part_floats) return hipErrorInvalidValue;   // the scratch is too small for this cut
    switch ((a.B + 31) / 32) {
    case 1: e = launch_block<1, DT>(a, parts, steps_per_part, s); break;
    case 2: e = launch_block<2, DT>(a, parts, steps_per_part, s); break;
    case 3: e = launch_block<3, DT>(a, parts, steps_per_part, s); break;
    default: e = launch_block<4, DT>(a, parts, steps_per_part, s); break;
    }
    if (e != hipSuccess) return e;
    const int n_out = (a.K_dst ? 3 : 1) * a.d;
    const int64_t threads = (int64_t)a.B * (n_out / 4);
    hipLaunchKernelGGL(qkv_finish_kernel<DT>, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s,
                       a.part, parts, static_cast<const elem_t *>(a.bq), static_cast<const elem_t *>(a.bkv),
                       static_cast<elem_t *>(a.q_out), static_cast<elem_t *>(a.K_dst), static_cast<elem_t *>(a.V_dst),
                       a.B, a.d, n_out, a.n_heads, a.head_dim, a.L_cap, a.tok_pos, paged_dst(a));
    return hipGetLastError();
}

}  // namespace

hipError_t launch_qkv_current(const QkvArgs &a, hipStream_t s)
{
    if (a.B <= 0) return hipSuccess;
    if (a.B > kQkvMaxRows || a.d % 64 != 0 || a.d > 256 * 8 * kMaxVec) return hipErrorInvalidValue;
    if (a.block_table && (!a.seq_len || a.max_blocks <= 0 || a.blk_log2 < 4 || a.blk_log2 > 10 || a.P_kv < 0 || a.P_act < 0))
        return hipErrorInvalidValue;
    return a.dtype == 1 ? launch_dt<1>(a, s) : launch_dt<0>(a, s);
}

// Parts of the reduction axis (d / 64 steps): about two workgroups per compute unit when Q, K and V are produced
// (measured cold on d = 4096 .. 9216: more parts cost more in fp32 partial sums than they gain in parallelism,
// fewer leave the Q-only call with too few workgroups), at least 4 steps per part, no empty part.  The same cut
// is used when only Q is produced, so that q does not depend on whether K/V are asked for (the order of the
// fp32 sums is the same), and the scratch size is a function of d and the row count alone.
void qkv_parts(int d, int *parts, int *steps_per_part)
{
    const int steps = d / 64;
    const int blocks = (d + 127) / 128 + (2 * d + 127) / 128;
    int want = 512 / blocks;
    if (want > steps / 4) want = steps / 4;
    if (want < 1) want = 1;
    if (want > 16) want = 16;
    *steps_per_part = (steps + want - 1) / want;
    *parts = (steps + *steps_per_part - 1) / *steps_per_part;
}

}  // namespace hk
