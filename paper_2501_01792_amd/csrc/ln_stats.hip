// Row-parallel LayerNorm statistics for gfx950: one 64-lane wavefront per checkpoint row.
//
// The checkpoint is the decoder layer's input (Sec. 3.3), so the layer's pre-attention
// LayerNorm has to be applied before Eq. 7.  This kernel only produces the two fp32
// numbers per row that the projection kernel needs to normalise the row on the fly:
//     stats[r] = (rstd, -mean * rstd),   rstd = 1 / sqrt(var + eps), var biased.
// Mean and variance are taken in two passes over the row (over a register copy of the row when it
// fits, else over memory, where the second pass hits L2), both summed in fp32 with wavefront shuffles.
#include "hk_internal.h"
#include "elem.h"

namespace hk {
namespace {

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

constexpr int kRowsPerBlock = 4;   // 256 threads = 4 wavefronts
constexpr int kMaxVec = 20;        // rows of up to 64 * 8 * 20 = 10240 elements are held in registers

// Rows that fit in registers are read from memory once: 16-byte loads, all issued before the first
// use, then mean and centred sum of squares from the register copy.
template <int DT, int NV>
__global__ __launch_bounds__(256) void ln_stats_reg_kernel(const typename Elem<DT>::T *__restrict__ act,
                                                           float2 *__restrict__ stats,
                                                           int64_t M, int d, float eps)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
    if (row >= M) return;   // whole wavefront leaves together; no barrier in this kernel
    typedef typename Elem<DT>::V8 half8_t;
    const half8_t *p = reinterpret_cast<const half8_t *>(act + row * (int64_t)d);
    const int nvec = d >> 3;   // host guarantees d % 8 == 0
    half8_t v[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int idx = lane + 64 * i;
        half8_t z;
#pragma unroll
        for (int j = 0; j < 8; ++j) z[j] = (typename Elem<DT>::T)0.f;
        v[i] = idx < nvec ? p[idx] : z;
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j) s += (float)v[i][j];
    const float mean = wave_sum(s) / (float)d;
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        if (lane + 64 * i < nvec) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float c = (float)v[i][j] - mean;
                ss += c * c;
            }
        }
    }
    const float var = wave_sum(ss) / (float)d;
    const float rstd = 1.0f / sqrtf(var + eps);
    if (lane == 0) stats[row] = make_float2(rstd, -mean * rstd);
}

// Any row length: two passes over memory (the second one hits L2).
template <int DT>
__global__ __launch_bounds__(256) void ln_stats_kernel(const typename Elem<DT>::T *__restrict__ act,
                                                       float2 *__restrict__ stats,
                                                       int64_t M, int d, float eps)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * kRowsPerBlock + (threadIdx.x >> 6);
    if (row >= M) return;   // whole wavefront leaves together; no barrier in this kernel
    typedef typename Elem<DT>::V8 half8_t;
    const half8_t *p = reinterpret_cast<const half8_t *>(act + row * (int64_t)d);
    const int nvec = d >> 3;

    float s = 0.f;
    for (int i = lane; i < nvec; i += 64) {
        const half8_t v = p[i];
#pragma unroll
        for (int j = 0; j < 8; ++j) s += (float)v[j];
    }
    const float mean = wave_sum(s) / (float)d;

    float ss = 0.f;
    for (int i = lane; i < nvec; i += 64) {
        const half8_t v = p[i];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float c = (float)v[j] - mean;
            ss += c * c;
        }
    }
    const float var = wave_sum(ss) / (float)d;
    const float rstd = 1.0f / sqrtf(var + eps);
    if (lane == 0) stats[row] = make_float2(rstd, -mean * rstd);
}

template <int DT>
hipError_t launch_dt(const void *act, float2 *stats, int64_t M, int d, float eps, hipStream_t s)
{
    const int64_t blocks = (M + kRowsPerBlock - 1) / kRowsPerBlock;
    const typename Elem<DT>::T *a = static_cast<const typename Elem<DT>::T *>(act);
    const int nv = (d / 8 + 63) / 64;          // 16-byte chunks per lane
    const dim3 grid((unsigned)blocks), block(256);
    if (nv <= 4) hipLaunchKernelGGL((ln_stats_reg_kernel<DT, 4>), grid, block, 0, s, a, stats, M, d, eps);
    else if (nv <= 8) hipLaunchKernelGGL((ln_stats_reg_kernel<DT, 8>), grid, block, 0, s, a, stats, M, d, eps);
    else if (nv <= 12) hipLaunchKernelGGL((ln_stats_reg_kernel<DT, 12>), grid, block, 0, s, a, stats, M, d, eps);
    else if (nv <= kMaxVec) hipLaunchKernelGGL((ln_stats_reg_kernel<DT, kMaxVec>), grid, block, 0, s, a, stats, M, d, eps);
    else hipLaunchKernelGGL(ln_stats_kernel<DT>, grid, block, 0, s, a, stats, M, d, eps);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_ln_stats(const void *act, float2 *stats, int64_t M, int d, float eps, hipStream_t s, int dtype)
{
    if (M <= 0) return hipSuccess;
    return dtype == 1 ? launch_dt<1>(act, stats, M, d, eps, s) : launch_dt<0>(act, stats, M, d, eps, s);
}

}  // namespace hk
