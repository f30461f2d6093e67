// "KV Gen" (Sec. 4.2.2; Eq. 7) for gfx950 with prepared layer weights: the LayerNorm is folded
// around the matrix product so that the main loop is a pure fp16 GEMM fed by direct-to-LDS loads.
//
// With  xhat_k = (x_k - mean) * rstd * gamma_k + beta_k  the projection of one token is
//     sum_k xhat_k W[n,k] + b[n]
//   = rstd * sum_k x_k (gamma_k W[n,k])  -  mean * rstd * sum_k gamma_k W[n,k]  +  (b[n] + sum_k beta_k W[n,k])
//   = rstd * (x . W'[n,:]) + nmr * c[n] + b'[n],            nmr = -mean * rstd,
// where W' = gamma-scaled weights (fp16), c[n] = sum_k W'[n,k] and b'[n] are per-layer constants
// produced once by prepare_layer (they depend on the layer's parameters only), and rstd, nmr are
// the per-row statistics of ln_stats.  The raw fp16 checkpoint rows feed the matrix cores as
// they are; the row statistics enter in the epilogue, in fp32.
//
// Kernel shape (CDNA4): 256 x 256 output tile, 4 wavefronts (128 x 128 accumulators each, in
// AGPRs), k advanced 32 at a time through a ring of 5 LDS stages (activations 16 KiB + weights
// 16 KiB each = 160 KiB).  Both operands are fetched with buffer_load ... lds (16 bytes per lane,
// a wavefront fills 16 consecutive 64-byte rows), four stages ahead of their use; the XOR
// swizzle of the 16-byte chunk index is applied on the global side.  No operand passes through
// a vector register before its fragment read, and the only vector-memory waits are the explicit
// per-step "stage kt+1 has landed" waits.  Fragments are double-buffered in registers; every
// MFMA slot carries at most one LDS read or one direct load.
#include "hk_internal.h"
#include "kv_gemm_common.h"

namespace hk {
namespace {

using namespace gemm;

constexpr int FBM = 256, FBN = 256, FBK = 32;
constexpr int FNT = 256;                                    // 4 wavefronts, 2 x 2
constexpr int FWM = 128, FWN = 128, FTM = 4, FTN = 4;
constexpr int kStages = 5;
constexpr int kOperandBytes = 256 * FBK * 2;                // 16 KiB: one operand of one stage
constexpr int kRingStageBytes = 2 * kOperandBytes;          // 32 KiB
constexpr int kRingBytes = kStages * kRingStageBytes;       // 160 KiB
constexpr int kRowBytes = FBK * 2;                          // 64-byte LDS rows, 4 chunks of 16 bytes
constexpr int kDmaPerStage = 8;                             // direct loads one lane issues per stage (4 + 4)
constexpr int kAhead = 4;                                   // stages in flight ahead of the one being consumed
// At the per-step wait, stages kt+2 .. kt+4 (3 x 8 loads) may still be in flight.
#define HK_FOLD_WAIT_NEXT_STAGE() asm volatile("s_waitcnt vmcnt(24)" ::: "memory")
static_assert((kAhead - 1) * kDmaPerStage == 24, "the wait above is written for 24 loads in flight");
// Inside a step the wait sits after 4 of the step's 8 loads: stages kt+2, kt+3 and half of kt+4 may fly.
#define HK_FOLD_WAIT_IN_STEP() asm volatile("s_waitcnt vmcnt(20)" ::: "memory")

typedef __attribute__((address_space(3))) void *lds_ptr_t;

struct Frags {
    half8_t a[FTM], b[FTN];
};

template <int GROUP_M>
__global__ __launch_bounds__(FNT) void kv_gemm_fold_kernel(
    const _Float16 *__restrict__ act, const float2 *__restrict__ stats,
    const _Float16 *__restrict__ Wp, const float *__restrict__ cvec, const float *__restrict__ bvec,
    _Float16 *__restrict__ K_out, _Float16 *__restrict__ V_out,
    int64_t M, int d, int n_heads, int head_dim, int L_act, int L_cap, int tok_off,
    int tiles_m, int tiles_n)
{
    extern __shared__ __align__(16) unsigned char smem[];

    const int N = 2 * d;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;

    int tile_m, tile_n;
    tile_coords<GROUP_M>(blockIdx.x, tiles_m, tiles_n, tile_m, tile_n);
    const int64_t m0 = (int64_t)tile_m * FBM;
    const int n0 = tile_n * FBN;

    // ---- direct-load roles.  The i-th load of a wavefront fills LDS rows 64 i + 16 wave .. + 15 of an
    // operand stage; lane l writes row (l / 4), physical chunk (l % 4), so it fetches the logical
    // chunk (l % 4) ^ ((row / 4) % 4) of that row: a ds_read_b128 is served 16 lanes (256 bytes, 64
    // banks) at a time, and 16 consecutive rows of one logical chunk then fall into 16 distinct slots.
    const int dr = lane >> 2;                                  // row inside the 16-row group
    const int dchunk = (lane & 3) ^ ((lane >> 4) & 3);         // logical 16-byte chunk to fetch
    int a_voff[4], b_voff[4];                                  // byte offsets from the tile bases
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int rho = 64 * i + 16 * wave + dr;
        int64_t m = m0 + rho;
        if (m >= M) m = M - 1;                                 // clamp: rows past the end are computed, never stored
        a_voff[i] = ((int)(m - m0) * d + dchunk * 8) * 2;
        int n = n0 + weight_row_of_lds_row<FWN, FTN>(rho);
        if (n >= N) n = N - 1;
        b_voff[i] = ((n - n0) * d + dchunk * 8) * 2;
    }
    const _Float16 *a_base = act + m0 * (int64_t)d;
    const _Float16 *b_base = Wp + (int64_t)n0 * d;
    int64_t a_bytes = (M - m0) * (int64_t)d * 2, b_bytes = ((int64_t)N - n0) * d * 2;
    if (a_bytes > 0x7fffffff) a_bytes = 0x7fffffff;            // a tile spans < 2^23 bytes
    if (b_bytes > 0x7fffffff) b_bytes = 0x7fffffff;
    const __amdgpu_buffer_rsrc_t a_rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<_Float16 *>(a_base), 0, (int)a_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t b_rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<_Float16 *>(b_base), 0, (int)b_bytes, 0x00020000);
    const int dma_wave = 16 * wave * kRowBytes;                // + 64 i rows, + stage, + operand

    // ---- fragment reads: row (lane % 32) + 32 i of the wavefront's sub-tile, chunk 2 ks + lane / 32
    const int fr = lane & 31, fc = lane >> 5;
    int frag_off[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) frag_off[ks] = fr * kRowBytes + (((2 * ks + fc) ^ ((fr >> 2) & 3)) << 4);
    const int a_rd_wave = wm * FWM * kRowBytes;
    const int b_rd_wave = kOperandBytes + wn * FWN * kRowBytes;

    const int nk = d / FBK;                                    // host guarantees d % 64 == 0
    // k offset of stage s; stages past the end wrap to valid addresses and are never consumed
    auto k_of_stage = [&](int s) { while (s >= nk) s -= nk; return s * FBK; };

    // j = 0..3: activations, j = 4..7: weights, of the stage at k offset k0 into ring slot `slot`
    auto issue_dma = [&](int k0, int slot, int j) {
        unsigned char *dst = smem + slot * kRingStageBytes + dma_wave + (j & 3) * (64 * kRowBytes);
        if (j < 4)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rsrc, (lds_ptr_t)dst, 16, a_voff[j], k0 * 2, 0, 0);
        else
            __builtin_amdgcn_raw_ptr_buffer_load_lds(b_rsrc, (lds_ptr_t)(dst + kOperandBytes), 16, b_voff[j - 4], k0 * 2, 0, 0);
    };
    // which = 0..3: a[which], 4..7: b[which - 4]
    auto read_frag = [&](Frags &f, int slot, int ks, int which) {
        const unsigned char *base = smem + slot * kRingStageBytes + frag_off[ks];
        if (which < 4)
            f.a[which] = *reinterpret_cast<const half8_t *>(base + a_rd_wave + which * (32 * kRowBytes));
        else
            f.b[which - 4] = *reinterpret_cast<const half8_t *>(base + b_rd_wave + (which - 4) * (32 * kRowBytes));
    };

    float16_t acc[FTM][FTN];
#pragma unroll
    for (int i = 0; i < FTM; ++i)
#pragma unroll
        for (int j = 0; j < FTN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    Frags f0, f1;

    // ---- prologue: stages 0 .. 3 in flight, stage 0 landed, its first fragments read
#pragma unroll
    for (int s = 0; s < kAhead; ++s) {
        const int k0 = k_of_stage(s);
#pragma unroll
        for (int j = 0; j < kDmaPerStage; ++j) issue_dma(k0, s, j);
    }
    HK_FOLD_WAIT_NEXT_STAGE();
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int q = 0; q < 8; ++q) read_frag(f0, 0, 0, q);

    int slot = 0;                                              // ring slot of stage kt
    for (int kt = 0; kt < nk; ++kt) {
        const int k4 = k_of_stage(kt + kAhead);
        const int slot1 = slot + 1 == kStages ? 0 : slot + 1;
        const int slot4 = slot + kAhead >= kStages ? slot + kAhead - kStages : slot + kAhead;
        // ---- P0: MFMAs of sub-step 0 (f0); fragments of sub-step 1 -> f1; one direct load of stage kt+4 every 4th slot
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            acc[q >> 2][q & 3] = __builtin_amdgcn_mfma_f32_32x32x16_f16(f0.a[q >> 2], f0.b[q & 3], acc[q >> 2][q & 3], 0, 0, 0);
            if (q < 8) read_frag(f1, slot, 1, q);
            if ((q & 3) == 3) issue_dma(k4, slot4, q >> 2);          // activations of stage kt+4
            __builtin_amdgcn_sched_barrier(0);
        }
        // ---- P1: MFMAs of sub-step 1 (f1); the step's wait + barrier; fragments of sub-step 0 of stage kt+1 -> f0
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            acc[q >> 2][q & 3] = __builtin_amdgcn_mfma_f32_32x32x16_f16(f1.a[q >> 2], f1.b[q & 3], acc[q >> 2][q & 3], 0, 0, 0);
            if (q == 1) {
                // Every LDS read of stage kt has been issued (P0).  Wait for them and for this
                // wavefront's loads of stage kt+1, then meet the others: after the barrier stage kt+1
                // is complete in LDS and the slot of stage kt may be refilled (by stage kt+5, next step).
                HK_FOLD_WAIT_IN_STEP();
                asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
            }
            if (q >= 2 && q < 10) read_frag(f0, slot1, 0, q - 2);
            if ((q & 3) == 3) issue_dma(k4, slot4, 4 + (q >> 2));    // weights of stage kt+4
            __builtin_amdgcn_sched_barrier(0);
        }
        slot = slot1;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");           // drain the loads issued past the end before LDS is released

    // ---- epilogue: LayerNorm statistics, constants of the layer, fp16, head split
    __syncthreads();                                           // every wavefront is done with the ring
    RowDst *tab = reinterpret_cast<RowDst *>(smem);
    fill_row_table<FBM, FNT>(tab, tid, m0, M, n_heads, head_dim, L_act, L_cap, tok_off, stats);
    const int nb = n0 + wn * FWN + FTN * (lane & 31);
    float cn[FTN], bn[FTN];
#pragma unroll
    for (int j = 0; j < FTN; ++j) {
        cn[j] = nb < N ? cvec[nb + j] : 0.f;
        bn[j] = nb < N ? bvec[nb + j] : 0.f;
    }
    __syncthreads();
    store_head_split<FTM, FTN>(acc, lane, tab, wm * FWM, nb, d, head_dim, L_cap, cn, bn, K_out, V_out);
}

// One wavefront per output feature n: W'[n,:] = fp16(gamma * W[n,:]), c[n] = sum_k W'[n,k],
// b'[n] = b[n] + sum_k beta_k W[n,k]  (sums in fp32).
__global__ __launch_bounds__(256) void prepare_layer_kernel(const _Float16 *__restrict__ W,
                                                            const _Float16 *__restrict__ bkv,
                                                            const _Float16 *__restrict__ ln_w,
                                                            const _Float16 *__restrict__ ln_b,
                                                            _Float16 *__restrict__ Wp, float *__restrict__ cvec,
                                                            float *__restrict__ bvec, int N, int d)
{
    const int lane = threadIdx.x & 63;
    const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (n >= N) return;                                        // whole wavefront leaves together; no barrier here
    const half8_t *src = reinterpret_cast<const half8_t *>(W + (int64_t)n * d);
    half8_t *dst = reinterpret_cast<half8_t *>(Wp + (int64_t)n * d);
    const half8_t *g = reinterpret_cast<const half8_t *>(ln_w);
    const half8_t *be = reinterpret_cast<const half8_t *>(ln_b);
    float c = 0.f, bb = 0.f;
    for (int i = lane; i < (d >> 3); i += 64) {
        const half8_t w = src[i], gv = g[i], bv = be[i];
        half8_t o;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            o[j] = (_Float16)((float)w[j] * (float)gv[j]);
            c += (float)o[j];
            bb = __builtin_fmaf((float)bv[j], (float)w[j], bb);
        }
        dst[i] = o;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        c += __shfl_xor(c, off, 64);
        bb += __shfl_xor(bb, off, 64);
    }
    if (lane == 0) {
        cvec[n] = c;
        bvec[n] = (float)bkv[n] + bb;
    }
}

}  // namespace

hipError_t launch_prepare_layer(const void *Wkv, const void *bkv, const void *ln_w, const void *ln_b,
                                void *Wp, float *cvec, float *bvec, int d, hipStream_t s)
{
    const int N = 2 * d;
    hipLaunchKernelGGL(prepare_layer_kernel, dim3((unsigned)((N + 3) / 4)), dim3(256), 0, s,
                       static_cast<const _Float16 *>(Wkv), static_cast<const _Float16 *>(bkv),
                       static_cast<const _Float16 *>(ln_w), static_cast<const _Float16 *>(ln_b),
                       static_cast<_Float16 *>(Wp), cvec, bvec, N, d);
    return hipGetLastError();
}

hipError_t launch_kv_gemm_fold(const KvGemmArgs &a, hipStream_t s)
{
    const int64_t tiles_m64 = (a.M + FBM - 1) / FBM;
    const int tiles_n = (2 * a.d + FBN - 1) / FBN;
    if (tiles_m64 * tiles_n > 0x7fffffffLL) return hipErrorInvalidValue;
    const int tiles_m = (int)tiles_m64;
    auto kern = kv_gemm_fold_kernel<4>;
    static_assert(kRingBytes == 160 * 1024, "the ring uses the whole 160 KiB LDS of a CU");
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kRingBytes);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)(tiles_m * tiles_n)), dim3(FNT), kRingBytes, s,
                       static_cast<const _Float16 *>(a.act), a.stats,
                       static_cast<const _Float16 *>(a.Wp), a.cvec, a.bvec,
                       static_cast<_Float16 *>(a.K_out), static_cast<_Float16 *>(a.V_out),
                       a.M, a.d, a.n_heads, a.head_dim, a.L_act, a.L_cap, a.tok_off, tiles_m, tiles_n);
    return hipGetLastError();
}

}  // namespace hk
