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
// bytes): an HBM streaming kernel.  Two kernels:
//   ln_rows:   one wavefront per row: statistics from a register copy of the row, then the normalised
//              row in fp16 to scratch (and the raw row to the checkpoint store when asked).
//   qkv_rows:  one workgroup per slab of 32 output features.  Its 4 wavefronts each take a quarter of
//              the reduction axis, stream their part of the 32 weight rows straight from HBM into
//              registers with whole-line loads (8 lanes per 128-byte line, several steps in flight),
//              turn them into MFMA operand layout through a private 4 KiB LDS block and multiply them
//              with the matching part of xhat (read through L2 the same way) on the matrix cores
//              (v_mfma_f32_32x32x16_f16).  The four partial sums meet in LDS; bias, fp16 and the
//              scatter to q / K / V follow.
#include "hk_internal.h"
#include "skinny_mma.h"

namespace hk {
namespace {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

constexpr int kMaxVec = 20;              // rows of up to 64 * 8 * 20 = 10240 elements are held in registers

// xhat[r, :] = ((x[r, :] - mean) * rstd) * gamma + beta in fp32, rounded once to fp16.
template <int NV>
__global__ __launch_bounds__(256) void ln_rows_kernel(const _Float16 *__restrict__ x, const _Float16 *__restrict__ gamma,
                                                      const _Float16 *__restrict__ beta, _Float16 *__restrict__ xhat,
                                                      _Float16 *__restrict__ act_dst, int64_t act_row_stride,
                                                      int B, int d, float eps)
{
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= B) return;                // whole wavefront leaves together; no barrier in this kernel
    const half8_t *p = reinterpret_cast<const half8_t *>(x + (int64_t)row * d);
    const int nvec = d >> 3;
    half8_t v[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int idx = lane + 64 * i;
        v[i] = idx < nvec ? p[idx] : half8_t{0, 0, 0, 0, 0, 0, 0, 0};
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) s += (float)v[i][j];
    const float mean = wave_sum(s) / (float)d;
    float sq = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        if (lane + 64 * i < nvec) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float c = (float)v[i][j] - mean;
                sq = __builtin_fmaf(c, c, sq);
            }
        }
    }
    const float rstd = 1.0f / __builtin_sqrtf(wave_sum(sq) / (float)d + eps);
    half8_t *dst = reinterpret_cast<half8_t *>(xhat + (int64_t)row * d);
    half8_t *ckpt = act_dst ? reinterpret_cast<half8_t *>(act_dst + (int64_t)row * act_row_stride) : nullptr;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int idx = lane + 64 * i;
        if (idx < nvec) {
            const half8_t g = reinterpret_cast<const half8_t *>(gamma)[idx], be = reinterpret_cast<const half8_t *>(beta)[idx];
            half8_t o;
#pragma unroll
            for (int j = 0; j < 8; ++j)
                o[j] = (_Float16)__builtin_fmaf(((float)v[i][j] - mean) * rstd, (float)g[j], (float)be[j]);
            dst[idx] = o;
            if (ckpt) ckpt[idx] = v[i];
        }
    }
}

using skinny::kSlab;

// RB = row blocks of 32 (B <= 32 RB)
template <int RB>
__global__ __launch_bounds__(256) void qkv_rows_kernel(
    const _Float16 *__restrict__ xhat, const _Float16 *__restrict__ Wq, const _Float16 *__restrict__ bq,
    const _Float16 *__restrict__ Wkv, const _Float16 *__restrict__ bkv,
    _Float16 *__restrict__ q_out, _Float16 *__restrict__ K_dst, _Float16 *__restrict__ V_dst,
    int B, int d, int n_heads, int head_dim, int L_cap, int tok_pos)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    const int n0 = blockIdx.x * kSlab;                     // first output feature of the slab, in [0, 3d)
    // the slab lies inside one of the three weight blocks (d % 32 == 0)
    const _Float16 *W = n0 < d ? Wq + (int64_t)n0 * d : Wkv + (int64_t)(n0 - d) * d;
    float (*red)[RB * 32][kSlab] = skinny::slab_product<RB, true>(W, kSlab, d, xhat, B, d, d, smem);

    // bias, fp16, scatter: thread -> (row, feature) pairs of the B x 32 slab
    const int which = n0 / d;                              // 0: q, 1: k, 2: v
    const int nn0 = n0 - which * d;
    for (int idx = tid; idx < B * kSlab; idx += 256) {
        const int m = idx / kSlab, c = idx % kSlab;
        const float sum = (red[0][m][c] + red[1][m][c]) + (red[2][m][c] + red[3][m][c]);
        const int nn = nn0 + c;
        const float bias = which == 0 ? (float)bq[nn] : (float)bkv[(which - 1) * d + nn];
        const _Float16 o = (_Float16)(sum + bias);
        if (which == 0) {
            q_out[(int64_t)m * d + nn] = o;
        } else {
            const int h = nn / head_dim, e = nn % head_dim;
            _Float16 *dst = which == 1 ? K_dst : V_dst;
            dst[(((int64_t)m * n_heads + h) * L_cap + tok_pos) * head_dim + e] = o;
        }
    }
}

template <int NV>
hipError_t launch_ln_rows(const QkvArgs &a, hipStream_t s)
{
    hipLaunchKernelGGL(ln_rows_kernel<NV>, dim3((unsigned)((a.B + 3) / 4)), dim3(256), 0, s,
                       static_cast<const _Float16 *>(a.x), static_cast<const _Float16 *>(a.ln_w),
                       static_cast<const _Float16 *>(a.ln_b), static_cast<_Float16 *>(a.xhat),
                       static_cast<_Float16 *>(a.act_dst), a.act_row_stride, a.B, a.d, a.eps);
    return hipGetLastError();
}

template <int RB>
hipError_t launch_rows(const QkvArgs &a, hipStream_t s)
{
    const int slabs = (a.K_dst ? 3 : 1) * (a.d / kSlab);
    auto kern = qkv_rows_kernel<RB>;
    constexpr int lds = skinny::lds_bytes<RB>();
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)slabs), dim3(256), lds, s,
                       static_cast<const _Float16 *>(a.xhat), static_cast<const _Float16 *>(a.Wq),
                       static_cast<const _Float16 *>(a.bq), static_cast<const _Float16 *>(a.Wkv),
                       static_cast<const _Float16 *>(a.bkv), static_cast<_Float16 *>(a.q_out),
                       static_cast<_Float16 *>(a.K_dst), static_cast<_Float16 *>(a.V_dst),
                       a.B, a.d, a.n_heads, a.head_dim, a.L_cap, a.tok_pos);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_qkv_current(const QkvArgs &a, hipStream_t s)
{
    if (a.B <= 0) return hipSuccess;
    if (a.B > kQkvMaxRows || a.d % 64 != 0 || a.d > 64 * 8 * kMaxVec) return hipErrorInvalidValue;
    hipError_t e;
    const int nv = (a.d / 8 + 63) / 64;
    if (nv <= 4) e = launch_ln_rows<4>(a, s);
    else if (nv <= 8) e = launch_ln_rows<8>(a, s);
    else if (nv <= 12) e = launch_ln_rows<12>(a, s);
    else if (nv <= 16) e = launch_ln_rows<16>(a, s);
    else e = launch_ln_rows<kMaxVec>(a, s);
    if (e != hipSuccess) return e;
    const int rb = (a.B + 31) / 32;
    switch (rb) {
    case 1: return launch_rows<1>(a, s);
    case 2: return launch_rows<2>(a, s);
    case 3: return launch_rows<3>(a, s);
    default: return launch_rows<4>(a, s);
    }
}

}  // namespace hk
