// "KV Gen" (Sec. 4.2.2; Eq. 7) for gfx950: LayerNorm-fused K/V projection on the matrix cores.
//
//   [K V][m, n] = sum_k xhat[m, k] * Wkv[n, k] + bkv[n],   xhat = LayerNorm(act) row by row,
//
// an M x 2d x d GEMM whose two operands are both contiguous along the reduction axis k.
//
// Design (CDNA4, 64-lane wavefronts, v_mfma_f32_32x32x16_f16, fp32 accumulate):
//   * One workgroup = 4 wavefronts (one per SIMD) computes a BM x BN output tile; the
//     wavefronts form a 2 x 2 grid, each owning a (BM/2) x (BN/2) sub-tile held in
//     accumulator registers.
//   * The k loop advances 64 at a time through a double-buffered LDS stage.  Global loads
//     of step k+1 are in flight while the MFMAs of step k run; one barrier per step.
//   * LayerNorm is the prologue of the A operand: raw fp16 activations are normalised in
//     registers (fp32: fma(x, rstd, -mean*rstd) * gamma + beta) on their way into LDS, so
//     the normalised activations never exist in HBM.  Row statistics come from ln_stats.
//   * LDS rows are 64 halves (128 B); the 16-byte chunk index is XOR-ed with (row & 7) so
//     the MFMA operand reads (32 rows x one chunk per half-wavefront) spread over all banks.
//   * Head-split epilogue without an LDS transpose: MFMA column c of column block jn is
//     given the weight row n = base + TN*c + jn.  A lane then owns TN consecutive output
//     features of one token across its TN column blocks, adds the bias in fp32, converts to
//     fp16 and writes them with one TN*2-byte store; half a wavefront covers 32*TN
//     consecutive features, i.e. whole head rows of the [B, H, L, dh] layout.
//   * Workgroup -> tile mapping: consecutive workgroup ids land on different XCDs, so ids
//     are first regrouped per XCD and then walked in column-major bands of GROUP_M row
//     tiles; the workgroups resident on one XCD share weight panels in that XCD's L2.
#include "hk_internal.h"

namespace hk {
namespace {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef float float16_t __attribute__((ext_vector_type(16)));

constexpr int BK = 64;            // k extent of one LDS stage (halves)
constexpr int kThreads = 256;
constexpr int kXcds = 8;

// Bijective regrouping of workgroup ids so that the ids served by one XCD (id % 8) become a
// contiguous range of tile numbers.
__host__ __device__ inline int xcd_regroup(int pid, int n)
{
    const int per = n / kXcds, rem = n % kXcds;   // the first `rem` XCDs serve per+1 tiles
    const int xcd = pid % kXcds, local = pid / kXcds;
    const int start = xcd * per + (xcd < rem ? xcd : rem);
    return start + local;
}

template <int BM, int BN>
struct __align__(16) Smem {
    _Float16 a[2][BM * BK];
    _Float16 b[2][BN * BK];
};

typedef uint32_t uint4_t __attribute__((ext_vector_type(4)));

// LayerNorm of two adjacent fp16 elements packed in one dword:
//   y = ((x * rstd + nmr) * gamma + beta),  nmr = -mean * rstd,
// as two mixed-precision FMAs per element (fp16 sources read in place, fp32 arithmetic, one
// rounding to fp16 on the way out).  Written with the instructions spelled out so that every
// element of every row takes the same rounding path wherever the row sits in a tile: the
// regenerated K/V of a token must not depend on which other tokens are regenerated with it.
__device__ __forceinline__ uint32_t ln_pair(uint32_t x, float rstd, float nmr, uint32_t gamma, uint32_t beta)
{
    float t0, t1;
    uint32_t y;
    asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel_hi:[1,0,0]" : "=v"(t0) : "v"(x), "v"(rstd), "v"(nmr));
    asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(t1) : "v"(x), "v"(rstd), "v"(nmr));
    asm("v_fma_mixlo_f16 %0, %1, %2, %3 op_sel_hi:[0,1,1]" : "=v"(y) : "v"(t0), "v"(gamma), "v"(beta));
    asm("v_fma_mixhi_f16 %0, %1, %2, %3 op_sel:[0,1,1] op_sel_hi:[0,1,1]" : "+v"(y) : "v"(t1), "v"(gamma), "v"(beta));
    return y;
}

// Byte-free index helpers for the swizzled [rows][64] half tiles.
__device__ __forceinline__ int lds_off(int row, int chunk) { return row * BK + ((chunk ^ (row & 7)) << 3); }

template <int BM, int BN, int GROUP_M>
__global__ __launch_bounds__(kThreads) void kv_gemm_kernel(const _Float16 *__restrict__ act,
                                                           const float2 *__restrict__ stats,
                                                           const _Float16 *__restrict__ ln_w,
                                                           const _Float16 *__restrict__ ln_b,
                                                           const _Float16 *__restrict__ Wkv,
                                                           const _Float16 *__restrict__ bkv,
                                                           _Float16 *__restrict__ K_out,
                                                           _Float16 *__restrict__ V_out,
                                                           int64_t M, int d, int n_heads, int head_dim,
                                                           int L_act, int L_cap, int tok_off,
                                                           int tiles_m, int tiles_n)
{
    constexpr int WM = BM / 2, WN = BN / 2;      // per-wavefront sub-tile
    constexpr int TM = WM / 32, TN = WN / 32;    // 32x32 MFMA blocks per wavefront
    constexpr int A_ITERS = BM / 32, B_ITERS = BN / 32;   // 16-byte chunks per thread per stage
    static_assert(TN == 2 || TN == 4, "epilogue packs TN halves per store");

    extern __shared__ __align__(16) unsigned char smem_raw[];
    Smem<BM, BN> &sm = *reinterpret_cast<Smem<BM, BN> *>(smem_raw);

    const int N = 2 * d;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // ---- tile assignment
    int tile_m, tile_n;
    {
        const int n_tiles = tiles_m * tiles_n;
        const int t = xcd_regroup(blockIdx.x, n_tiles);
        const int band = GROUP_M * tiles_n;
        const int g = t / band;
        const int first_m = g * GROUP_M;
        const int rows = (tiles_m - first_m < GROUP_M) ? (tiles_m - first_m) : GROUP_M;
        const int in = t - g * band;
        tile_m = first_m + in % rows;
        tile_n = in / rows;
    }
    const int64_t m0 = (int64_t)tile_m * BM;
    const int n0 = tile_n * BN;

    // ---- global -> LDS assignment: thread handles chunk column `lc` of rows lr + 32*i
    const int lc = tid & 7;
    const int lr = tid >> 3;

    const _Float16 *a_ptr[A_ITERS];
    float2 a_stat[A_ITERS];
#pragma unroll
    for (int i = 0; i < A_ITERS; ++i) {
        int64_t m = m0 + lr + 32 * i;
        if (m >= M) m = M - 1;                    // clamp: rows past the end are computed, never stored
        a_ptr[i] = act + m * (int64_t)d + lc * 8;
        a_stat[i] = stats[m];
    }
    const _Float16 *b_ptr[B_ITERS];
#pragma unroll
    for (int i = 0; i < B_ITERS; ++i) {
        const int rho = lr + 32 * i;              // LDS row of the weight tile
        const int w = rho / WN, r = rho % WN;     // owning wavefront column, row inside it
        int n = n0 + w * WN + TN * (r & 31) + (r >> 5);
        if (n >= N) n = N - 1;
        b_ptr[i] = Wkv + (int64_t)n * d + lc * 8;
    }

    half8_t a_raw[A_ITERS], b_raw[B_ITERS], g_raw, be_raw;

    auto load_stage = [&](int k0) {
#pragma unroll
        for (int i = 0; i < A_ITERS; ++i) a_raw[i] = *reinterpret_cast<const half8_t *>(a_ptr[i] + k0);
#pragma unroll
        for (int i = 0; i < B_ITERS; ++i) b_raw[i] = *reinterpret_cast<const half8_t *>(b_ptr[i] + k0);
        g_raw = *reinterpret_cast<const half8_t *>(ln_w + k0 + lc * 8);
        be_raw = *reinterpret_cast<const half8_t *>(ln_b + k0 + lc * 8);
    };
    auto store_stage = [&](int buf) {
        const uint4_t g = __builtin_bit_cast(uint4_t, g_raw), be = __builtin_bit_cast(uint4_t, be_raw);
#pragma unroll
        for (int i = 0; i < A_ITERS; ++i) {
            const uint4_t x = __builtin_bit_cast(uint4_t, a_raw[i]);
            uint4_t y;
#pragma unroll
            for (int w = 0; w < 4; ++w) y[w] = ln_pair(x[w], a_stat[i].x, a_stat[i].y, g[w], be[w]);
            *reinterpret_cast<uint4_t *>(&sm.a[buf][lds_off(lr + 32 * i, lc)]) = y;
        }
#pragma unroll
        for (int i = 0; i < B_ITERS; ++i)
            *reinterpret_cast<half8_t *>(&sm.b[buf][lds_off(lr + 32 * i, lc)]) = b_raw[i];
    };

    float16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int nk = d / BK;                         // host guarantees d % 64 == 0
    load_stage(0);
    store_stage(0);
    __syncthreads();

    const int frag_row = lane & 31;
    const int frag_chunk = lane >> 5;
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) load_stage((kt + 1) * BK);
        const _Float16 *sa = sm.a[buf] + (wm * WM) * BK;
        const _Float16 *sb = sm.b[buf] + (wn * WN) * BK;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            half8_t af[TM], bf[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                af[i] = *reinterpret_cast<const half8_t *>(&sa[lds_off(i * 32 + frag_row, ks * 2 + frag_chunk)]);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                bf[j] = *reinterpret_cast<const half8_t *>(&sb[lds_off(j * 32 + frag_row, ks * 2 + frag_chunk)]);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[i], bf[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) store_stage(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: bias, fp16, head split.  Lane owns features nb .. nb+TN-1.
    const int nb = n0 + wn * WN + TN * (lane & 31);
    if (nb < N) {                                  // N % TN == 0, so the group is all in or all out
        float bias[TN];
#pragma unroll
        for (int j = 0; j < TN; ++j) bias[j] = (float)bkv[nb + j];
        const bool is_v = nb >= d;
        const int nn = is_v ? nb - d : nb;
        const int h = nn / head_dim, e = nn % head_dim;
        _Float16 *dst_base = (is_v ? V_out : K_out) + e;
        // (sequence, token) of the tile's first row, once per workgroup; rows below it are
        // reached by adding the row offset and carrying into the sequence index.
        const uint32_t b0 = (uint32_t)m0 / (uint32_t)L_act, t0 = (uint32_t)m0 % (uint32_t)L_act;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int dm = wm * WM + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
                const int64_t m = m0 + dm;
                if (m < M) {
                    uint32_t b = b0, t = t0 + (uint32_t)dm;
                    if (L_act >= BM) {                    // at most one carry inside a tile
                        if (t >= (uint32_t)L_act) { t -= (uint32_t)L_act; ++b; }
                    } else {
                        b += t / (uint32_t)L_act;
                        t %= (uint32_t)L_act;
                    }
                    _Float16 *dst = dst_base + (((int64_t)b * n_heads + h) * (int64_t)L_cap + tok_off + t) * head_dim;
                    if constexpr (TN == 4) {
                        half4_t v;
#pragma unroll
                        for (int j = 0; j < 4; ++j) v[j] = (_Float16)(acc[i][j][r] + bias[j]);
                        *reinterpret_cast<half4_t *>(dst) = v;
                    } else {
                        half2_t v;
#pragma unroll
                        for (int j = 0; j < 2; ++j) v[j] = (_Float16)(acc[i][j][r] + bias[j]);
                        *reinterpret_cast<half2_t *>(dst) = v;
                    }
                }
            }
        }
    }
}

template <int BM, int BN, int GROUP_M>
hipError_t launch_tile(const KvGemmArgs &a, hipStream_t s)
{
    const int64_t tiles_m64 = (a.M + BM - 1) / BM;
    const int tiles_n = (2 * a.d + BN - 1) / BN;
    if (tiles_m64 * tiles_n > 0x7fffffffLL) return hipErrorInvalidValue;
    const int tiles_m = (int)tiles_m64;
    auto kern = kv_gemm_kernel<BM, BN, GROUP_M>;
    constexpr size_t smem = sizeof(Smem<BM, BN>);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)(tiles_m * tiles_n)), dim3(kThreads), smem, s,
                       static_cast<const _Float16 *>(a.act), a.stats,
                       static_cast<const _Float16 *>(a.ln_w), static_cast<const _Float16 *>(a.ln_b),
                       static_cast<const _Float16 *>(a.Wkv), static_cast<const _Float16 *>(a.bkv),
                       static_cast<_Float16 *>(a.K_out), static_cast<_Float16 *>(a.V_out),
                       a.M, a.d, a.n_heads, a.head_dim, a.L_act, a.L_cap, a.tok_off, tiles_m, tiles_n);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_kv_gemm(const KvGemmArgs &a, hipStream_t s)
{
    if (a.M <= 0) return hipSuccess;
    // Large problems: 256x256 tiles (highest reuse per LDS byte).  Problems with too few such
    // tiles to occupy the 256 compute units fall back to 128x128 tiles.
    const int64_t big_tiles = ((a.M + 255) / 256) * ((2 * (int64_t)a.d + 255) / 256);
    const int tile = a.tile ? a.tile : (big_tiles >= 512 ? 256 : 128);
    if (tile == 256) return launch_tile<256, 256, 8>(a, s);
    return launch_tile<128, 128, 8>(a, s);
}

}  // namespace hk
