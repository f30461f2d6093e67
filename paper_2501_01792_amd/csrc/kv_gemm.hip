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
//   (This is the kernel for small problems; large ones take the streaming kernel of kv_gemm_fold.hip.)
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
#include "kv_gemm_common.h"

namespace hk {
namespace {

using namespace gemm;

template <int BM, int BN, int WAVES_M, int WAVES_N, int GROUP_M>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N) void kv_gemm_kernel(
    const _Float16 *__restrict__ act, const float2 *__restrict__ stats,
    const _Float16 *__restrict__ ln_w, const _Float16 *__restrict__ ln_b,
    const _Float16 *__restrict__ Wkv, const _Float16 *__restrict__ bkv,
    _Float16 *__restrict__ K_out, _Float16 *__restrict__ V_out,
    int64_t M, int d, int n_heads, int head_dim, int L_act, int L_cap, int tok_off,
    int tiles_m, int tiles_n)
{
    constexpr int NT = 64 * WAVES_M * WAVES_N;             // threads per workgroup
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;    // per-wavefront sub-tile
    constexpr int TM = WM / 32, TN = WN / 32;              // 32x32 MFMA blocks per wavefront
    constexpr int LROWS = NT / 8;                          // tile rows covered by one pass of 16-byte loads
    constexpr int A_ITERS = BM / LROWS, B_ITERS = BN / LROWS;
    static_assert(TN == 1 || TN == 2 || TN == 4, "epilogue packs TN halves per store");
    static_assert(BM % LROWS == 0 && BN % LROWS == 0, "tile rows must split evenly over the loader threads");

    extern __shared__ __align__(16) unsigned char smem_raw[];
    Smem<BM, BN> &sm = *reinterpret_cast<Smem<BM, BN> *>(smem_raw);

    const int N = 2 * d;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WAVES_N, wn = wave % WAVES_N;

    int tile_m, tile_n;
    tile_coords<GROUP_M>(blockIdx.x, tiles_m, tiles_n, tile_m, tile_n);
    const int64_t m0 = (int64_t)tile_m * BM;
    const int n0 = tile_n * BN;

    // ---- global -> LDS assignment: thread handles chunk column `lc` of rows lr + LROWS*i
    const int lc = tid & 7;
    const int lr = tid >> 3;

    const _Float16 *a_ptr[A_ITERS];
    float2 a_stat[A_ITERS];
#pragma unroll
    for (int i = 0; i < A_ITERS; ++i) {
        int64_t m = m0 + lr + LROWS * i;
        if (m >= M) m = M - 1;                    // clamp: rows past the end are computed, never stored
        a_ptr[i] = act + m * (int64_t)d + lc * 8;
        a_stat[i] = stats[m];
    }
    const _Float16 *b_ptr[B_ITERS];
#pragma unroll
    for (int i = 0; i < B_ITERS; ++i) {
        int n = n0 + weight_row_of_lds_row<WN, TN>(lr + LROWS * i);
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
            *reinterpret_cast<uint4_t *>(&sm.a[buf][lds_off(lr + LROWS * i, lc)]) = y;
        }
#pragma unroll
        for (int i = 0; i < B_ITERS; ++i)
            *reinterpret_cast<half8_t *>(&sm.b[buf][lds_off(lr + LROWS * i, lc)]) = b_raw[i];
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

    // ---- epilogue: bias, fp16, head split (the loop's last barrier has retired every read of the stages)
    RowDst *tab = reinterpret_cast<RowDst *>(smem_raw);
    fill_row_table<BM, 64 * WAVES_M * WAVES_N>(tab, tid, m0, M, n_heads, head_dim, L_act, L_cap, tok_off, nullptr);
    const int nb = n0 + wn * WN + TN * (lane & 31);
    float cn[TN], bn[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        cn[j] = 0.f;
        bn[j] = nb < 2 * d ? (float)bkv[nb + j] : 0.f;
    }
    __syncthreads();
    store_head_split<TM, TN>(acc, lane, tab, wm * WM, nb, d, head_dim, L_cap, cn, bn, K_out, V_out);
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int GROUP_M>
hipError_t launch_tile(const KvGemmArgs &a, hipStream_t s)
{
    const int64_t tiles_m64 = (a.M + BM - 1) / BM;
    const int tiles_n = (2 * a.d + BN - 1) / BN;
    if (tiles_m64 * tiles_n > 0x7fffffffLL) return hipErrorInvalidValue;
    const int tiles_m = (int)tiles_m64;
    auto kern = kv_gemm_kernel<BM, BN, WAVES_M, WAVES_N, GROUP_M>;
    constexpr size_t smem = sizeof(Smem<BM, BN>);
    static LdsOnce lds_once;
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kern), (int)smem, lds_once);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)(tiles_m * tiles_n)), dim3(64 * WAVES_M * WAVES_N), smem, s,
                       static_cast<const _Float16 *>(a.act), a.stats,
                       static_cast<const _Float16 *>(a.ln_w), static_cast<const _Float16 *>(a.ln_b),
                       static_cast<const _Float16 *>(a.Wkv), static_cast<const _Float16 *>(a.bkv),
                       static_cast<_Float16 *>(a.K_out), static_cast<_Float16 *>(a.V_out),
                       a.M, a.d, a.n_heads, a.head_dim, a.L_act, a.L_cap, a.tok_off, tiles_m, tiles_n);
    return hipGetLastError();
}

}  // namespace

bool kv_gemm_uses_prepared(int64_t M, int d, int tile, int dtype)
{
    if (dtype == 1) return true;                           // bf16: one kernel for every problem size
    // Large problems: 256x256 tiles (highest reuse per LDS byte).  Problems with too few such
    // tiles to occupy the 256 compute units take 128x128 tiles.
    const int64_t big_tiles = ((M + 255) / 256) * ((2 * (int64_t)d + 255) / 256);
    return (tile ? tile : (big_tiles >= 512 ? 256 : 128)) == 256;
}

hipError_t launch_kv_gemm(const KvGemmArgs &a, hipStream_t s)
{
    if (a.M <= 0) return hipSuccess;
    if (kv_gemm_uses_prepared(a.M, a.d, a.tile, a.dtype)) {
        if (!a.Wp || !a.cvec || !a.bvec) return hipErrorInvalidValue;
        return launch_kv_gemm_fold(a, s);                  // LayerNorm folded around the product
    }
    return launch_tile<128, 128, 2, 2, 8>(a, s);           // LayerNorm as the GEMM prologue
}

}  // namespace hk
