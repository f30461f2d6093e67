// "KV Gen" (Sec. 4.2.2; Eq. 7) for gfx950, large-problem kernel: 256 x 256 output tiles,
// 4 wavefronts (one per SIMD, 128 x 128 accumulators each), software-pipelined over three
// stages of the reduction axis.
//
// Same computation and output layout as the generic kernel in kv_gemm.hip; what differs is how
// the operands reach the matrix cores.  One k step (64) of a 256 x 256 tile is under a
// microsecond of MFMA time, so a global load issued and consumed within one step exposes the
// memory latency at every step.  Here every load is issued two steps ahead of its use, and the
// instruction stream of a step is laid out by hand around its 64 MFMAs:
//
//   step kt, phase 0..3 (one k sub-step of 16 = 16 MFMAs each), fragments double-buffered:
//     P0  issue loads of stage kt+2: weights straight into LDS (buffer_load ... lds, buffer (kt+2)%3),
//         activations + LayerNorm weight/bias into registers (set kt&1);
//         read fragments of sub-step 1;  MFMAs of sub-step 0;  LayerNorm of stage kt+1, part 1
//     P1  read fragments of sub-step 2;  MFMAs of sub-step 1;  LayerNorm of stage kt+1, part 2
//     P2  read fragments of sub-step 3;  MFMAs of sub-step 2;  LayerNorm of stage kt+1, part 3;
//         wait: weights of stage kt+1 landed, own LDS traffic done;  barrier
//     P3  read fragments of sub-step 0 of stage kt+1;  MFMAs of sub-step 3
//
// Weights never pass through registers: each wavefront's 16-byte-per-lane direct loads fill
// 8 consecutive LDS rows (1 KiB), and the XOR swizzle of the chunk index is applied on the
// global side (a lane fetches the chunk that belongs in its LDS slot).  Activations do pass
// through registers because the LayerNorm prologue is applied there, once per element, on the
// way into LDS.  LDS: 2 activation buffers + 3 weight buffers of 32 KiB = 160 KiB.
#include "hk_internal.h"
#include "kv_gemm_common.h"

namespace hk {
namespace {

using namespace gemm;

constexpr int PBM = 256, PBN = 256;
constexpr int PWAVES_M = 2, PWAVES_N = 2;
constexpr int PNT = 64 * PWAVES_M * PWAVES_N;               // 256 threads
constexpr int PWM = PBM / PWAVES_M, PWN = PBN / PWAVES_N;   // 128 x 128 per wavefront
constexpr int PTM = PWM / 32, PTN = PWN / 32;               // 4 x 4 MFMA blocks
constexpr int PLROWS = PNT / 8;                             // 32 tile rows per pass of 16-byte loads
constexpr int PA_ITERS = PBM / PLROWS;                      // 8 activation chunks per lane per stage
constexpr int PB_ITERS = PBN / PLROWS;                      // 8 direct weight loads per lane per stage
constexpr int kStageHalves = 256 * BK;                      // one operand stage, in halves
constexpr int kStageBytes = kStageHalves * 2;               // 32 KiB
constexpr int kLoadsPerStage = PA_ITERS + PB_ITERS + 2;     // vector-memory operations one lane issues per stage
static_assert(kLoadsPerStage == 18, "the waits below are written for 18 loads per stage");
#define HK_WAIT_STAGE_LANDED() asm volatile("s_waitcnt vmcnt(18)" ::: "memory")

// LDS map (bytes): activations [0, 64 KiB) as two stages, weights [64 KiB, 160 KiB) as three.
constexpr int kLdsA = 0, kLdsB = 2 * kStageBytes, kLdsTotal = 5 * kStageBytes;

typedef __attribute__((address_space(3))) void *lds_ptr_t;
typedef const __attribute__((address_space(1))) void *global_ptr_t;

struct Frags {
    half8_t a[PTM], b[PTN];
};

template <int GROUP_M>
__global__ __launch_bounds__(PNT) void kv_gemm_pipe_kernel(
    const _Float16 *__restrict__ act, const float2 *__restrict__ stats,
    const _Float16 *__restrict__ ln_w, const _Float16 *__restrict__ ln_b,
    const _Float16 *__restrict__ Wkv, const _Float16 *__restrict__ bkv,
    _Float16 *__restrict__ K_out, _Float16 *__restrict__ V_out,
    int64_t M, int d, int n_heads, int head_dim, int L_act, int L_cap, int tok_off,
    int tiles_m, int tiles_n)
{
    extern __shared__ __align__(16) unsigned char smem[];

    const int N = 2 * d;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / PWAVES_N, wn = wave % PWAVES_N;

    int tile_m, tile_n;
    tile_coords<GROUP_M>(blockIdx.x, tiles_m, tiles_n, tile_m, tile_n);
    const int64_t m0 = (int64_t)tile_m * PBM;
    const int n0 = tile_n * PBN;

    // ---- loader roles.  lc: 16-byte chunk column, lr: row within a 32-row pass.
    const int lc = tid & 7;
    const int lr = tid >> 3;

    // activations: rows lr + 32 i, logical chunk lc.  Addresses are a wave-uniform tile base plus a
    // 32-bit per-lane offset (a tile spans < 2^22 halves), which keeps them in one VGPR each.
    const _Float16 *a_base = act + m0 * (int64_t)d;
    uint32_t a_off[PA_ITERS];
    float2 a_stat[PA_ITERS];
#pragma unroll
    for (int i = 0; i < PA_ITERS; ++i) {
        int64_t m = m0 + lr + PLROWS * i;
        if (m >= M) m = M - 1;                    // clamp: rows past the end are computed, never stored
        a_off[i] = (uint32_t)(m - m0) * (uint32_t)d + lc * 8;
        a_stat[i] = stats[m];
    }
    // weights: LDS slot (row lr + 32 i, physical chunk lc) <- logical chunk lc ^ (row & 7) of that row's weight row
    const _Float16 *b_base = Wkv + (int64_t)n0 * d;
    uint32_t b_off[PB_ITERS];
#pragma unroll
    for (int i = 0; i < PB_ITERS; ++i) {
        const int rho = lr + PLROWS * i;
        int n = n0 + weight_row_of_lds_row<PWN, PTN>(rho);
        if (n >= N) n = N - 1;
        b_off[i] = (uint32_t)(n - n0) * (uint32_t)d + ((lc ^ (rho & 7)) << 3);
    }
    // LDS byte offsets.  A store slot of this lane inside a stage; wave-uniform start of the 8 rows
    // (1 KiB) that this wavefront's i-th direct load fills.
    const int a_st_off = lr * (BK * 2) + ((lc ^ (lr & 7)) << 4);   // + i * 32 rows * 128 B
    const int b_dma_wave = wave * 8 * (BK * 2);                    // + i * 32 rows * 128 B
    // fragment reads: row (lane % 32) + 32 i of the wavefront's sub-tile, chunk 2 ks + lane / 32
    const int fr = lane & 31, fc = lane >> 5;
    int frag_off[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) frag_off[ks] = fr * (BK * 2) + (((2 * ks + fc) ^ (fr & 7)) << 4);
    const int a_rd_wave = kLdsA + wm * PWM * (BK * 2);
    const int b_rd_wave = kLdsB + wn * PWN * (BK * 2);

    const int nk = d / BK;                        // host guarantees d % 64 == 0
    const int k_last = (nk - 1) * BK;

    // Two register sets for the activations in flight; every use names its set with a
    // compile-time constant so that the sets stay in registers.
    struct RawSet {
        half8_t a[PA_ITERS], g, be;
    } raw0, raw1;

    // stage -> where its weights go: `bslot` cycles 0,1,2 with the stage number
    // Direct-to-LDS loads go through a buffer resource over the rest of the weight matrix: that
    // form is counted in order with the other vector loads, so waits can be exact.
    const __amdgpu_buffer_rsrc_t b_rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<_Float16 *>(b_base), 0, (int)(((int64_t)N - n0) * d * 2), 0x00020000);
    auto issue_weight_load = [&](int k0, int bslot, int i) {
        unsigned char *dst = smem + kLdsB + bslot * kStageBytes + b_dma_wave + i * (PLROWS * BK * 2);
        __builtin_amdgcn_raw_ptr_buffer_load_lds(b_rsrc, (lds_ptr_t)dst, 16, (int)(b_off[i] * 2), k0 * 2, 0, 0);
    };
    auto issue_act_load = [&](int k0, RawSet &r, int i) {
        r.a[i] = *reinterpret_cast<const half8_t *>(a_base + k0 + a_off[i]);
    };
    auto issue_ln_param_loads = [&](int k0, RawSet &r) {
        r.g = *reinterpret_cast<const half8_t *>(ln_w + k0 + lc * 8);
        r.be = *reinterpret_cast<const half8_t *>(ln_b + k0 + lc * 8);
    };
    // LayerNorm of one dword (two elements) of chunk i; the chunk is stored once its 4 dwords are done.
    uint4_t ln_y;
    auto ln_quarter = [&](const RawSet &r, int abuf, int i, int w) {
        const uint4_t g = __builtin_bit_cast(uint4_t, r.g), be = __builtin_bit_cast(uint4_t, r.be);
        const uint4_t x = __builtin_bit_cast(uint4_t, r.a[i]);
        ln_y[w] = ln_pair(x[w], a_stat[i].x, a_stat[i].y, g[w], be[w]);
        if (w == 3)
            *reinterpret_cast<uint4_t *>(smem + kLdsA + abuf * kStageBytes + a_st_off + i * (PLROWS * BK * 2)) = ln_y;
    };
    auto read_frags = [&](Frags &f, int abuf, int bslot, int ks, int which) {
        // which: 0..3 -> a[which], 4..7 -> b[which - 4]
        if (which < 4)
            f.a[which] = *reinterpret_cast<const half8_t *>(smem + a_rd_wave + abuf * kStageBytes + frag_off[ks] + which * (32 * BK * 2));
        else
            f.b[which - 4] = *reinterpret_cast<const half8_t *>(smem + b_rd_wave + bslot * kStageBytes + frag_off[ks] + (which - 4) * (32 * BK * 2));
    };

    float16_t acc[PTM][PTN];
#pragma unroll
    for (int i = 0; i < PTM; ++i)
#pragma unroll
        for (int j = 0; j < PTN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    Frags f0, f1;

    // One k step.  ld: register set receiving stage kt+2; nx: register set holding stage kt+1.
    // bs: weight LDS slot of stage kt (slots of kt+1, kt+2 follow cyclically).
    auto step = [&](int kt, int bs, RawSet &ld, const RawSet &nx) {
        int k2 = (kt + 2) * BK;
        if (k2 > k_last) k2 = k_last;             // past the end: reload the last stage (never consumed)
        const int abuf = kt & 1, abuf_n = abuf ^ 1;
        const int bs1 = bs == 2 ? 0 : bs + 1, bs2 = bs1 == 2 ? 0 : bs1 + 1;
        // ---- P0: MFMAs of sub-step 0 (f0); loads of stage kt+2 (activations first: they are consumed
        //      first, by next step's LayerNorm); fragments of sub-step 1 -> f1; LN quarters 0..3
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            acc[q >> 2][q & 3] = __builtin_amdgcn_mfma_f32_32x32x16_f16(f0.a[q >> 2], f0.b[q & 3], acc[q >> 2][q & 3], 0, 0, 0);
            if (q < 8) read_frags(f1, abuf, bs, 1, q);
            if (q == 0) issue_ln_param_loads(k2, ld);
            if (q < 8) issue_act_load(k2, ld, q);
            if (q >= 8) issue_weight_load(k2, bs2, q - 8);
            if (q >= 12) ln_quarter(nx, abuf_n, 0, q - 12);
            __builtin_amdgcn_sched_barrier(0);
        }
        // ---- P1: MFMAs of sub-step 1 (f1); fragments of sub-step 2 -> f0; LN quarters 4..19
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            acc[q >> 2][q & 3] = __builtin_amdgcn_mfma_f32_32x32x16_f16(f1.a[q >> 2], f1.b[q & 3], acc[q >> 2][q & 3], 0, 0, 0);
            if (q < 8) read_frags(f0, abuf, bs, 2, q);
            ln_quarter(nx, abuf_n, 1 + (q >> 2), q & 3);
            __builtin_amdgcn_sched_barrier(0);
        }
        // ---- P2: MFMAs of sub-step 2 (f0); fragments of sub-step 3 -> f1; LN quarters 20..31; then the step's barrier
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            acc[q >> 2][q & 3] = __builtin_amdgcn_mfma_f32_32x32x16_f16(f0.a[q >> 2], f0.b[q & 3], acc[q >> 2][q & 3], 0, 0, 0);
            if (q < 8) read_frags(f1, abuf, bs, 3, q);
            if (q < 12) ln_quarter(nx, abuf_n, 5 + (q >> 2), q & 3);
            __builtin_amdgcn_sched_barrier(0);
            if (q == 11) {
                // All LDS reads of stage kt are issued and all writes of stage kt+1 are issued; wait for
                // them and for the weights of stage kt+1 (issued one step ago: only this step's 18 loads
                // may still be in flight), then meet the other wavefronts.
                HK_WAIT_STAGE_LANDED();
                asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // ---- P3: MFMAs of sub-step 3 (f1); fragments of sub-step 0 of stage kt+1 -> f0
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            acc[q >> 2][q & 3] = __builtin_amdgcn_mfma_f32_32x32x16_f16(f1.a[q >> 2], f1.b[q & 3], acc[q >> 2][q & 3], 0, 0, 0);
            if (q < 8) read_frags(f0, abuf_n, bs1, 0, q);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ---- prologue: stages 0 and 1 in flight, stage 0 normalised into LDS, first fragments read
    {
        int k1 = BK > k_last ? k_last : BK;
        issue_ln_param_loads(0, raw0);
#pragma unroll
        for (int i = 0; i < PA_ITERS; ++i) issue_act_load(0, raw0, i);
#pragma unroll
        for (int i = 0; i < PB_ITERS; ++i) issue_weight_load(0, 0, i);
        issue_ln_param_loads(k1, raw1);
#pragma unroll
        for (int i = 0; i < PA_ITERS; ++i) issue_act_load(k1, raw1, i);
#pragma unroll
        for (int i = 0; i < PB_ITERS; ++i) issue_weight_load(k1, 1, i);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < PA_ITERS; ++i)
#pragma unroll
            for (int w = 0; w < 4; ++w) ln_quarter(raw0, 0, i, w);
        HK_WAIT_STAGE_LANDED();                   // all of stage 0 has landed (the 18 loads of stage 1 may fly)
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int q = 0; q < 8; ++q) read_frags(f0, 0, 0, 0, q);
    }

    int kt = 0, bs = 0;
    for (; kt + 1 < nk; kt += 2) {
        step(kt, bs, raw0, raw1);
        bs = bs == 2 ? 0 : bs + 1;
        step(kt + 1, bs, raw1, raw0);
        bs = bs == 2 ? 0 : bs + 1;
    }
    if (kt < nk) step(kt, bs, raw0, raw1);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");       // drain the loads issued past the end before LDS is released

    __syncthreads();                                       // every wavefront is done with the stages
    RowDst *tab = reinterpret_cast<RowDst *>(smem);
    fill_row_table<PBM, PNT>(tab, tid, m0, M, n_heads, head_dim, L_act, L_cap, tok_off, nullptr);
    const int nb = n0 + wn * PWN + PTN * (lane & 31);
    float cn[PTN], bn[PTN];
#pragma unroll
    for (int j = 0; j < PTN; ++j) {
        cn[j] = 0.f;
        bn[j] = nb < 2 * d ? (float)bkv[nb + j] : 0.f;
    }
    __syncthreads();
    store_head_split<PTM, PTN>(acc, lane, tab, wm * PWM, nb, d, head_dim, L_cap, cn, bn, K_out, V_out);
}

}  // namespace

hipError_t launch_kv_gemm_pipe(const KvGemmArgs &a, hipStream_t s)
{
    const int64_t tiles_m64 = (a.M + PBM - 1) / PBM;
    const int tiles_n = (2 * a.d + PBN - 1) / PBN;
    if (tiles_m64 * tiles_n > 0x7fffffffLL) return hipErrorInvalidValue;
    const int tiles_m = (int)tiles_m64;
    auto kern = kv_gemm_pipe_kernel<8>;
    static_assert(kLdsTotal == 160 * 1024, "the pipeline uses the whole 160 KiB LDS of a CU");
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, kLdsTotal);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)(tiles_m * tiles_n)), dim3(PNT), kLdsTotal, s,
                       static_cast<const _Float16 *>(a.act), a.stats,
                       static_cast<const _Float16 *>(a.ln_w), static_cast<const _Float16 *>(a.ln_b),
                       static_cast<const _Float16 *>(a.Wkv), static_cast<const _Float16 *>(a.bkv),
                       static_cast<_Float16 *>(a.K_out), static_cast<_Float16 *>(a.V_out),
                       a.M, a.d, a.n_heads, a.head_dim, a.L_act, a.L_cap, a.tok_off, tiles_m, tiles_n);
    return hipGetLastError();
}

}  // namespace hk
