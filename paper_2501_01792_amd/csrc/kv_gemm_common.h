// Device helpers shared by the K/V projection kernels (tile addressing, LDS swizzle, the
// LayerNorm prologue arithmetic).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hk {
namespace gemm {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef float float16_t __attribute__((ext_vector_type(16)));

constexpr int BK = 64;            // k extent of one LDS stage (halves)
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

// Workgroup id -> output tile.  Ids are regrouped per XCD, then tiles are walked in bands of
// GROUP_M row tiles, column-major inside a band, so that the workgroups resident on one XCD
// at a time share a few activation row panels and weight column panels in that XCD's L2.
template <int GROUP_M>
__device__ __forceinline__ void tile_coords(int pid, int tiles_m, int tiles_n, int &tile_m, int &tile_n)
{
    const int t = xcd_regroup(pid, tiles_m * tiles_n);
    const int band = GROUP_M * tiles_n;
    const int g = t / band;
    const int first_m = g * GROUP_M;
    const int rows = (tiles_m - first_m < GROUP_M) ? (tiles_m - first_m) : GROUP_M;
    const int in = t - g * band;
    tile_m = first_m + in % rows;
    tile_n = in / rows;
}

// Weight row held by LDS row `rho` of a BN-row weight tile.  MFMA column c of column block jn
// of wavefront column w is given output feature w*WN + TN*c + jn, so that a lane ends up with
// TN consecutive features of one token across its TN accumulator blocks.
template <int WN, int TN>
__device__ __forceinline__ int weight_row_of_lds_row(int rho)
{
    const int w = rho / WN, r = rho % WN;
    return w * WN + TN * (r & 31) + (r >> 5);
}

// Where a token row of an output tile goes, and the LayerNorm statistics that its accumulators
// are to be combined with.  One entry per tile row, built once per tile in LDS (the operand
// stages are dead by then) so that the store loop itself has no division, no global load and
// no divergent control flow.
struct __align__(16) RowDst {
    float rstd, nmr;      // (1, 0) when the accumulators already hold the projection of LayerNorm-ed rows
    int64_t base;         // element offset of K[b, 0, tok_off + t, 0]; negative: row is past the end, store nothing
};

// Table entry of global row m: where its head-split output starts and its LayerNorm statistics.
__device__ __forceinline__ RowDst row_dst(int64_t m, int64_t M, int n_heads, int head_dim, int L_act, int L_cap, int tok_off,
                                          const float2 *__restrict__ stats)
{
    RowDst e;
    e.rstd = 1.f; e.nmr = 0.f; e.base = -1;
    if (m < M) {
        const uint32_t b = (uint32_t)m / (uint32_t)L_act, t = (uint32_t)m % (uint32_t)L_act;   // M < 2^31
        e.base = (((int64_t)b * n_heads) * L_cap + tok_off + t) * head_dim;
        if (stats) { const float2 st = stats[m]; e.rstd = st.x; e.nmr = st.y; }
    }
    return e;
}

// Fills tab[0 .. BM) for the tile whose first row is m0.  Call between two workgroup barriers.
template <int BM, int NT>
__device__ __forceinline__ void fill_row_table(RowDst *tab, int tid, int64_t m0, int64_t M,
                                               int n_heads, int head_dim, int L_act, int L_cap, int tok_off,
                                               const float2 *__restrict__ stats)
{
    for (int row = tid; row < BM; row += NT) tab[row] = row_dst(m0 + row, M, n_heads, head_dim, L_act, L_cap, tok_off, stats);
}

// The stores are non-temporal: the regenerated rows are read once, by the attention kernel, and must
// not linger as dirty lines in the last-level cache, where their write-back would compete with that
// kernel's reads.
// Epilogue of one wavefront: out = rstd * acc + (nmr * cn + bn) in fp32, round to fp16, head-split
// store into [B, H, L_cap, dh].  With the row table's (rstd, nmr) = (1, 0) this is acc + bn, the plain
// bias add; with the row statistics it is the folded LayerNorm (cn = c[n], bn = b'[n]).
// acc[i][j][r] is MFMA block (i, j), register r: tile row wrow0 + 32 i + 8 (r/4) + 4 (lane/32) + r%4,
// output feature nb + j with nb = n0 + wcol0 + TN * (lane % 32).
template <int TM, int TN>
__device__ __forceinline__ void store_head_split(const float16_t (&acc)[TM][TN], int lane, const RowDst *tab,
                                                 int wrow0, int nb, int d, int head_dim, int L_cap,
                                                 const float (&cn)[TN], const float (&bn)[TN],
                                                 _Float16 *__restrict__ K_out, _Float16 *__restrict__ V_out)
{
    if (nb >= 2 * d) return;                       // 2d % TN == 0: the lane's features are all in or all out
    const bool is_v = nb >= d;
    const int nn = is_v ? nb - d : nb;
    const int h = nn / head_dim, e = nn % head_dim;
    _Float16 *dst_base = (is_v ? V_out : K_out) + ((int64_t)h * L_cap * head_dim + e);
    const RowDst *my = tab + wrow0 + 4 * (lane >> 5);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const RowDst row = my[i * 32 + 8 * (r >> 2) + (r & 3)];
            if (row.base >= 0) {
                _Float16 *dst = dst_base + row.base;
                if constexpr (TN == 4) {
                    half4_t v;
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        v[j] = (_Float16)__builtin_fmaf(acc[i][j][r], row.rstd, __builtin_fmaf(row.nmr, cn[j], bn[j]));
                    __builtin_nontemporal_store(v, reinterpret_cast<half4_t *>(dst));
                } else if constexpr (TN == 2) {
                    half2_t v;
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        v[j] = (_Float16)__builtin_fmaf(acc[i][j][r], row.rstd, __builtin_fmaf(row.nmr, cn[j], bn[j]));
                    __builtin_nontemporal_store(v, reinterpret_cast<half2_t *>(dst));
                } else {
                    *dst = (_Float16)__builtin_fmaf(acc[i][0][r], row.rstd, __builtin_fmaf(row.nmr, cn[0], bn[0]));
                }
            }
        }
    }
}

}  // namespace gemm
}  // namespace hk
