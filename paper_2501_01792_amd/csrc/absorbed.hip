// Decode attention over the activation checkpoints WITHOUT regenerating their K/V rows.
//
// The hybrid step (Sec. 4.2.2) turns every checkpoint row x_t into a K row and a V row (Eq. 7) and then runs
// the single-query attention (Eq. 4) over them.  For one query per head the two linear maps can be moved to
// the other side of the sums, which gives the same result (up to rounding) for ~head_dim times fewer FLOP:
// with the folded LayerNorm  K_t = rstd_t (x_t W'_K^T) + nmr_t c_K + b'_K  (likewise V),
//
//   score_t(h) = scale [ rstd_t (x_t . u_h - mean_t sum_k u_h[k]) + q_h . b'_K,h ],     u_h = q_h W'_K,h   [d]
//   o_h        = W'_V,h y_h + b'_V,h,            y_h = sum_t w_t (x_t - mean_t),         w_t = p_t rstd_t / l
//
// so the checkpoints are streamed twice (scores, weighted row sum) and the weights once; nothing of size
// [tokens, 2 d] is ever written.  u_h, w_t and y_h are kept in fp16; the two mean terms are formed from the
// ROUNDED values (sum_k of the stored u_h, sum_t of the stored w_t) and subtracted in fp32 before anything is
// rounded again, so that a row mean that is large against the row's spread cancels exactly as it does in
// the LayerNorm, instead of leaving the rounding error of u_h or w_t multiplied by it.  The cached K/V segment goes through the ordinary decode kernel and the two
// segments are joined by their softmax maxima and denominators.  Tensors stored as bfloat16 (q, the checkpoints, the
// prepared weights, the cached segment's output, out) are converted to fp16 where they are loaded, so the
// arithmetic, and with it the cancellation argument above, is the same for both storage types; u, w, y are fp16
// either way.  This is a comparison variant beyond the
// paper's design (which regenerates K/V with a GEMM); the paper's Eq. 3/4/7 define the result.
//
// Kernels (B sequences, H heads, L_act checkpoint rows per sequence):
//   carry   U[h,b,:]  = q[b,h,:] W'_K,h          rows of W' reduced       column_product (MFMA)
//   scores  raw[b,h,t] = x[b,t,:] . U[h,b,:]     rows of x streamed       skinny::slab_product, or block_product from
//                                                                         65536 rows on (MFMA); also the LayerNorm
//                                                                         statistics of the rows
//   softmax w[b,h,t]  = p_t rstd_t / l           one wavefront per (b,h)
//   gather  Y[b,h,:]  = sum_t w[b,h,t] x[b,t,:] - sum_t w[b,h,t] mean_t   rows of x reduced   column_product (MFMA)
//   project o[b,h,:]  = W'_V,h Y[b,h,:] + b'_V   rows of W' streamed      skinny::slab_product (MFMA), joins the cached part;
//                                                                         layers of 5120 features or more: block_product
//                                                                         with the reduction axis cut over workgroups, then
//                                                                         a join kernel
#include "hk_internal.h"
#include "kv_gemm_common.h"
#include "skinny_mma.h"

namespace hk {
namespace {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef short short4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) short4_t *lds_short4_ptr;

constexpr float kNegBig = -1.0e30f;

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

// ---------------------------------------------------------------------------------------------------------
// column_product: Out[z][m][c] = sum_r A[z][m][r] * S[z][r][c]   (m < a_rows <= 32 RB, r < R, c < n_cols)
//
// The streamed operand S is row-major and the reduction runs over its ROWS, so it reaches the matrix cores
// transposed.  Every wavefront owns a block of 64 columns and walks all R rows in steps of 16: whole 128-byte
// pieces of 16 rows go from HBM to registers (kDepth - 1 steps in flight) and row-wise into the wavefront's
// private LDS block, from which every lane takes the 8 values of its column with two transposing reads
// (ds_read_b64_tr_b16; rows 192 bytes apart, so that the four rows one such read touches fall on disjoint banks).  The small operand A (few rows, reduction axis contiguous, zero
// beyond R up to the next multiple of 64) is the same for the four wavefronts of a workgroup: it is fetched
// once per 64 reduction elements with whole-line loads, two tiles ahead, and shared through a double-buffered
// LDS tile (one barrier per 64 reduction elements).  The result (minus an optional per-row constant, in fp32)
// leaves through the private LDS block so that it is stored as whole 128-byte rows.
struct ColArgs {
    const _Float16 *S; int64_t s_batch, ld_s; int R, n_cols;
    const _Float16 *A; int64_t a_batch, ld_a; int a_rows;
    _Float16 *Out; int64_t o_batch, ld_out;
    const float *shift; int64_t shift_batch; int shift_stride;   // optional: Out[z][m][:] -= shift[z shift_batch + m shift_stride]
    // optional, for rows that live in blocks of 2^blk_log2 (>= 16) rows scattered over a pool: row r of batch z is
    // row r % block of pool block blk_list[z list_pitch + r / block] (S then points at the pool, s_batch = 0), and
    // batch z has R_list[z] rows (0: the output rows of z are zero)
    const int32_t *blk_list; int list_pitch, blk_log2;
    const int32_t *R_list;
    int s_dt, a_dt;                                        // storage types of S and of A (Out is fp16)
};

constexpr int kColBlock = 64;                              // columns of one wavefront
constexpr int kColPitch = 2 * kColBlock + 64;               // bytes between rows of a wavefront's private LDS block
constexpr int kColStage = 32 * kColPitch;                  // bytes of private LDS per wavefront
constexpr int kTileBytes = 32 * 128;                       // 32 operand rows x 64 reduction elements

template <int RB>
constexpr int col_lds_bytes() { return 4 * kColStage + 2 * RB * kTileBytes; }

template <int RB, int SDT, int ADT>
__global__ __launch_bounds__(256) void column_product_kernel(ColArgs p)
{
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int NB = kColBlock / 32;
    constexpr int XS = kColPitch;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    int c0 = (blockIdx.x * 4 + wave) * kColBlock;
    const bool live = c0 < p.n_cols;                       // a wavefront past the last column block works on the
    if (!live) c0 = p.n_cols - kColBlock;                  // last one (it shares the barriers) and stores nothing
    const int64_t z = blockIdx.y;
    const _Float16 *S = p.S + z * p.s_batch + c0;
    const _Float16 *A = p.A + z * p.a_batch;
    const int R = p.R_list ? p.R_list[z] : p.R;            // uniform over the workgroup
    const int steps = (R + 15) / 16;
    const int tiles = (steps + 3) / 4;

    // one load instruction: 8 rows x 128 bytes, 8 lanes per row
    const int g_row = lane >> 3, g_chunk = lane & 7;
    const int ln = lane & 31, lh = lane >> 5;
    // the A tile: thread -> (row tid / 8 of every 32-row block, 16-byte chunk tid % 8)
    const int t_row = tid >> 3, t_chunk = tid & 7;
    const _Float16 *ap[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        int m = rb * 32 + t_row;
        if (m >= p.a_rows) m = p.a_rows - 1;               // clamp: rows past the end are computed, never stored
        ap[rb] = A + (int64_t)m * p.ld_a + 8 * t_chunk;
    }
    // tile layout: row-major 128-byte rows, chunk index XOR-ed with (row / 2) % 8 (conflict-free both ways)
    const int t_wr = t_row * 128 + ((t_chunk ^ ((t_row >> 1) & 7)) << 4);
    int t_rd[4];                                           // operand fragment of step s % 4: chunks 2 (s % 4) + lane / 32
#pragma unroll
    for (int q = 0; q < 4; ++q) t_rd[q] = ln * 128 + (((2 * q + lh) ^ ((ln >> 1) & 7)) << 4);
    unsigned char *my = smem + wave * kColStage;
    unsigned char *tile = smem + 4 * kColStage;
    // source address of this lane in the transposing reads of the private block: lane 16 g + t points at row
    // 8 (g / 2) + t / 4, columns 16 (g % 2) + 4 (t % 4) .. + 3 (of column block nb: + 32 nb; second read: 4 rows on)
    const int tr_off = (8 * (lane >> 5) + ((lane & 15) >> 2)) * XS + 2 * (16 * ((lane >> 4) & 1) + 4 * (lane & 3));

    float16_t acc[RB][NB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[rb][nb][r] = 0.f;

    constexpr int kDepth = 8;                              // streamed steps in registers; two tiles per pass of the loop
    half8_t sv[kDepth][2];
    half8_t av[2][RB];
    const int last = steps - 1, last_tile = tiles - 1;
    auto clamp = [&](int sc) { return sc < last ? sc : last; };
    auto load_s = [&](int slot, int sc) {
        // the 16 rows of a step share a block; its number comes through a scalar load (sc and z are uniform), which
        // does not wait for the vector loads in flight
        const int r0 = 16 * sc;
        int64_t first = r0;
        if (p.blk_list) {
            const int32_t bid = p.blk_list[z * p.list_pitch + (r0 >> p.blk_log2)];
            first = ((int64_t)bid << p.blk_log2) + (r0 & ((1 << p.blk_log2) - 1));
        }
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            int rr = 8 * j + g_row;
            if (r0 + rr >= R) rr = R - 1 - r0;             // rows past the end meet zeros of A; r0 < R for every step asked for
            sv[slot][j] = *reinterpret_cast<const half8_t *>(S + (first + rr) * p.ld_s + 8 * g_chunk);
        }
    };
    auto load_a = [&](int slot, int g) {
        if (g > last_tile) g = last_tile;
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) av[slot][rb] = *reinterpret_cast<const half8_t *>(ap[rb] + 64 * g);
    };
    auto put_a = [&](int slot, int buf) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
            *reinterpret_cast<half8_t *>(tile + (buf * RB + rb) * kTileBytes + t_wr) = skinny::to_half8<ADT>(av[slot][rb]);
    };
    if (R <= 0) {                                          // nothing to sum (uniform over the workgroup: no barrier is missed)
        if (live) {
            _Float16 *Out0 = p.Out + z * p.o_batch + c0;
            half8_t zero8;
#pragma unroll
            for (int i = 0; i < 8; ++i) zero8[i] = (_Float16)0.f;
            for (int m = g_row; m < p.a_rows; m += 8) *reinterpret_cast<half8_t *>(Out0 + (int64_t)m * p.ld_out + 8 * g_chunk) = zero8;
        }
        return;
    }
    // Every load of the loop is unconditional (steps and tiles past the end re-read the last one), so that
    // the number of loads in flight at each wait is a compile-time fact.
    load_a(0, 0);
    load_a(1, 1);
#pragma unroll
    for (int u = 0; u < kDepth - 1; ++u) load_s(u, clamp(u));
    put_a(0, 0);
    __syncthreads();
    for (int g0 = 0; g0 < tiles; g0 += 2) {
#pragma unroll
        for (int gg = 0; gg < 2; ++gg) {
            const int g = g0 + gg;
            if (g < tiles) {                               // uniform over the workgroup
                put_a((gg + 1) & 1, (gg + 1) & 1);         // tile g + 1 (fetched one pass ago) for the next pass
                load_a(gg, g + 2);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int u = 4 * gg + q, sc = 4 * g + q;
                    load_s((u + kDepth - 1) % kDepth, clamp(sc + kDepth - 1));
                    if (sc < steps) {
#pragma unroll
                        for (int j = 0; j < 2; ++j)
                            *reinterpret_cast<half8_t *>(my + (8 * j + g_row) * XS + 16 * g_chunk) = skinny::to_half8<SDT>(sv[u][j]);
                        // bf[nb][i] = element (row 8 lh + i, column 32 nb + ln) of the block, by two transposing reads:
                        // ds_read_b64_tr_b16 hands lane t of a 16-lane group the four rows that the group's lanes
                        // 4 j + t / 4 .. point at, at column 4 (source lane % 4) + ... = t of the group's 16 columns
                        half8_t bf[NB];
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb) {
                            const short4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(my + tr_off + 64 * nb));
                            const short4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_short4_ptr)(my + tr_off + 64 * nb + 4 * XS));
                            bf[nb] = __builtin_bit_cast(half8_t, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                        }
#pragma unroll
                        for (int rb = 0; rb < RB; ++rb) {
                            const half8_t af = *reinterpret_cast<const half8_t *>(tile + (gg * RB + rb) * kTileBytes + t_rd[q]);
#pragma unroll
                            for (int nb = 0; nb < NB; ++nb)
                                acc[rb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af, bf[nb], acc[rb][nb], 0, 0, 0);
                        }
                    }
                }
                __syncthreads();                           // tile g + 1 is complete; tile g is free for g + 2
            }
        }
    }
    if (!live) return;                                     // no barrier below

    // ---- fp16, through the private LDS block, out as whole rows.
    // acc[rb][nb][r]: row 32 rb + 8 (r/4) + 4 (lane/32) + r%4, column 32 nb + lane%32.
    _Float16 *Out = p.Out + z * p.o_batch + c0;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        float sub[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            int m = 32 * rb + 8 * (r >> 2) + 4 * lh + (r & 3);
            if (m >= p.a_rows) m = p.a_rows - 1;
            sub[r] = p.shift ? p.shift[z * p.shift_batch + (int64_t)m * p.shift_stride] : 0.f;
        }
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                *reinterpret_cast<_Float16 *>(my + (8 * (r >> 2) + 4 * lh + (r & 3)) * XS + 2 * (32 * nb + ln)) =
                    (_Float16)(acc[rb][nb][r] - sub[r]);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int m = 32 * rb + 8 * j + g_row;
            const half8_t o = *reinterpret_cast<const half8_t *>(my + (8 * j + g_row) * XS + 16 * g_chunk);
            if (m < p.a_rows) *reinterpret_cast<half8_t *>(Out + (int64_t)m * p.ld_out + 8 * g_chunk) = o;
        }
    }
}

template <int RB, int SDT, int ADT>
hipError_t launch_col_as(const ColArgs &p, int batches, hipStream_t s)
{
    auto kern = column_product_kernel<RB, SDT, ADT>;
    constexpr int lds = col_lds_bytes<RB>();
    static LdsOnce lds_once;
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kern), lds, lds_once);
    if (e != hipSuccess) return e;
    const int blocks_x = (p.n_cols / kColBlock + 3) / 4;
    hipLaunchKernelGGL(kern, dim3((unsigned)blocks_x, (unsigned)batches), dim3(256), lds, s, p);
    return hipGetLastError();
}

template <int RB>
hipError_t launch_col(const ColArgs &p, int batches, hipStream_t s)
{
    if (p.s_dt == 0 && p.a_dt == 0) return launch_col_as<RB, 0, 0>(p, batches, s);
    if (p.s_dt == 1 && p.a_dt == 1) return launch_col_as<RB, 1, 1>(p, batches, s);
    if (p.s_dt == 1 && p.a_dt == 0) return launch_col_as<RB, 1, 0>(p, batches, s);
    return hipErrorInvalidValue;
}

// A must be readable (and zero beyond R) up to the next multiple of 64 reduction elements.
hipError_t launch_column_product(const ColArgs &p, int batches, hipStream_t s)
{
    if (p.a_rows <= 0 || p.a_rows > 128 || p.R <= 0 || p.n_cols % kColBlock != 0 || batches <= 0 || batches > 65535)
        return hipErrorInvalidValue;
    switch ((p.a_rows + 31) / 32) {
    case 1: return launch_col<1>(p, batches, s);
    case 2: return launch_col<2>(p, batches, s);
    case 3: return launch_col<3>(p, batches, s);
    default: return launch_col<4>(p, batches, s);
    }
}

// ---------------------------------------------------------------------------------------------------------
// scores: raw[b][h][t] = (x[b,t,:] - x[b,t,0]) . U[h,b,:] for the checkpoint rows of one sequence, and the
// LayerNorm statistics of those rows from the same pass:
//   stats[b L_act + t] = (rstd, mean, -(mean - x[b,t,0]) rstd, -)
// The rows enter the product minus their first element, so that a large row mean is neither multiplied with
// the rounding error of U nor left to cancel later.  Workgroup ids are regrouped so that the workgroups of one
// sequence, which share that sequence's U rows, run on one XCD and find them in its L2.
__device__ __forceinline__ float4 row_stats(float s1, float s2, float first, int d, float eps)
{
    const float inv_d = 1.0f / (float)d;
    const float dm = s1 * inv_d;                           // mean - first element
    const float var = fmaxf(__builtin_fmaf(-dm, dm, s2 * inv_d), 0.f);
    const float rstd = 1.0f / __builtin_sqrtf(var + eps);
    return make_float4(rstd, first + dm, -dm * rstd, 0.f);
}

// Few checkpoint rows in all: a slab of 32 rows per workgroup, the reduction axis cut over its 4 wavefronts
// (skinny::slab_product), so that even a small problem fills the chip.  Every workgroup reads all of U[:,b,:].
template <int RB, int DT>
__global__ __launch_bounds__(256) void absorbed_scores_kernel(const _Float16 *__restrict__ act, const _Float16 *__restrict__ U,
                                                              float *__restrict__ raw, float4 *__restrict__ stats,
                                                              int B, int L_act, int Lp, int H, int d, float eps)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    const int slabs = (L_act + skinny::kSlab - 1) / skinny::kSlab;
    const int item = gemm::xcd_regroup(blockIdx.x, slabs * B);
    const int64_t b = item / slabs;
    const int t0 = (item % slabs) * skinny::kSlab;
    const int rows = L_act - t0 < skinny::kSlab ? L_act - t0 : skinny::kSlab;
    const _Float16 *S = act + (b * L_act + t0) * d;
    float (*red)[RB * 32][skinny::kSlab] = skinny::slab_product<RB, false, true, DT>(S, rows, d, U + b * d, H, (int64_t)B * d, d, smem);
    for (int idx = tid; idx < H * skinny::kSlab; idx += 256) {
        const int h = idx / skinny::kSlab, c = idx % skinny::kSlab;
        if (c < rows)
            raw[(b * H + h) * Lp + t0 + c] = (red[0][h][c] + red[1][h][c]) + (red[2][h][c] + red[3][h][c]);
    }
    if (tid < rows) {
        float (*mom)[skinny::kSlab][2] = skinny::moments<RB>(smem);
        const float s1 = (mom[0][tid][0] + mom[1][tid][0]) + (mom[2][tid][0] + mom[3][tid][0]);
        const float s2 = (mom[0][tid][1] + mom[1][tid][1]) + (mom[2][tid][1] + mom[3][tid][1]);
        stats[b * L_act + t0 + tid] = row_stats(s1, s2, (float)skinny::stored_to_half<DT>(S + (int64_t)tid * d), d, eps);
    }
}

// Many checkpoint rows: 128 rows per workgroup (skinny::block_product): U is read once per 128 rows instead of
// once per 32, and scores and statistics are stored straight from registers.
template <int RB, int DT>
__global__ __launch_bounds__(256) void absorbed_scores_block_kernel(const _Float16 *__restrict__ act, const _Float16 *__restrict__ U,
                                                                    float *__restrict__ raw, float4 *__restrict__ stats,
                                                                    int B, int L_act, int Lp, int H, int d, float eps)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int blocks = (L_act + 127) / 128;
    const int item = gemm::xcd_regroup(blockIdx.x, blocks * B);
    const int64_t b = item / blocks;
    const int t0 = (item % blocks) * 128;
    const int tw = t0 + 32 * wave;                         // first row of this wavefront
    const int rows = L_act - tw < 32 ? (L_act - tw > 0 ? L_act - tw : 0) : 32;
    float16_t acc[RB];
    float m1[4], m2[4];
    _Float16 first[4];
    skinny::block_product<RB, false, true, DT>(act + (b * L_act + t0) * d, L_act - t0 < 128 ? L_act - t0 : 128, d,
                                           U + b * d, H, (int64_t)B * d, 0, d / 64, smem, acc, m1, m2, first);
    const int ln = lane & 31, lh = lane >> 5;
    if (ln < rows) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int h = 32 * rb + 8 * (r >> 2) + 4 * lh + (r & 3);
                if (h < H) raw[(b * H + h) * Lp + tw + ln] = acc[rb][r];
            }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int row = 8 * j + (lane >> 3);
        if ((lane & 7) == 0 && row < rows) stats[b * L_act + tw + row] = row_stats(m1[j], m2[j], (float)first[j], d, eps);
    }
}

// softmax over the checkpoint rows of one (sequence, head), one wavefront each.  In the log2 domain:
//   s_t = sl (rstd_t raw_t + k_t c1 + c2),  k_t = -(mean_t - x_t[0]) rstd_t,  c1 = q . c_K,h,  c2 = q . b'_K,h,
//   sl = scale log2(e);   w_t = fp16(2^(s_t - m) rstd_t / l), zero from L_act to the next multiple of 64;
//   sums = (m, l, sum_t w_t mean_t with the stored w_t, -)
template <int DT>
__global__ __launch_bounds__(256) void absorbed_softmax_kernel(const _Float16 *__restrict__ q,
                                                               const float *__restrict__ raw, const float4 *__restrict__ stats,
                                                               const float *__restrict__ cvec, const float *__restrict__ bvec,
                                                               _Float16 *__restrict__ w, float4 *__restrict__ sums,
                                                               int B, int H, int head_dim, int L_all, int Lp, float sl,
                                                               const int32_t *__restrict__ n_rows, int stats_pitch)
{
    const int lane = threadIdx.x & 63;
    const int bh = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (bh >= B * H) return;                               // whole wavefront leaves together; no barrier in this kernel
    const int b = bh / H, h = bh % H;
    const int L_act = n_rows ? n_rows[b] : L_all;          // sequences may have their own numbers of rows (0: no weight at all)
    float c1 = 0.f, c2 = 0.f;
    for (int e = lane; e < head_dim; e += 64) {
        const float qe = skinny::stored_to_float<DT>(q + (int64_t)bh * head_dim + e);
        c1 = __builtin_fmaf(qe, cvec[h * head_dim + e], c1);
        c2 = __builtin_fmaf(qe, bvec[h * head_dim + e], c2);
    }
    c1 = wave_sum(c1);
    c2 = wave_sum(c2);
    const float *r = raw + (int64_t)bh * Lp;
    const float4 *st = stats + (int64_t)b * stats_pitch;
    // Every load is unconditional (rows past the end re-read the last row and are masked afterwards) and loads come in
    // batches of kBatch rows per lane: a load under a per-row test makes the compiler wait for it before the next one
    // is issued, and the kernel then pays one memory latency per row and lane.
    const int t_last = L_act > 0 ? L_act - 1 : 0;          // row 0 of the scratch rows is readable even without rows
    constexpr int kBatch = 8;
    auto score_of = [&](const float4 &s4, float rv) { return sl * (__builtin_fmaf(s4.x, rv, __builtin_fmaf(s4.z, c1, c2))); };
    // The first 64 kKeep rows stay in registers (score, rstd, mean), so that up to that many rows are read once
    // (the statistics of a row are shared by all heads: re-reading them per pass made this kernel L2-bound);
    // rows beyond are read again in each of the three passes.  (Keeping 64 scores per lane and re-reading the
    // statistics in the last pass instead was slower: 57 against 32 us on 2048 rows, no faster on 4096.)
    constexpr int kKeep = 32;
    float sc[kKeep], rs[kKeep], mn[kKeep];
    float mx = kNegBig;
#pragma unroll
    for (int c = 0; c < kKeep; c += kBatch) {
        float4 s4[kBatch];
        float rv[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int t = lane + 64 * (c + u), tc = t < t_last ? t : t_last;
            s4[u] = st[tc];
            rv[u] = r[tc];
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const bool valid = lane + 64 * (c + u) < L_act;
            sc[c + u] = valid ? score_of(s4[u], rv[u]) : kNegBig;
            rs[c + u] = valid ? s4[u].x : 0.f;
            mn[c + u] = valid ? s4[u].y : 0.f;
            mx = fmaxf(mx, sc[c + u]);
        }
    }
    // rows beyond the kept ones, kBatch per lane at a time: fn(row, valid, score, rstd, mean)
    auto tail_rows = [&](auto fn, int end) {
        for (int t0 = lane + 64 * kKeep; t0 - lane < end; t0 += 64 * kBatch) {
            float4 s4[kBatch];
            float rv[kBatch];
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const int t = t0 + 64 * u, tc = t < t_last ? t : t_last;
                s4[u] = st[tc];
                rv[u] = r[tc];
            }
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const int t = t0 + 64 * u;
                fn(t, t < L_act, score_of(s4[u], rv[u]), s4[u].x, s4[u].y);
            }
        }
    };
    tail_rows([&](int, bool valid, float sv, float, float) { if (valid) mx = fmaxf(mx, sv); }, L_act);
    mx = wave_max(mx);
    float l = 0.f;
#pragma unroll
    for (int i = 0; i < kKeep; ++i)
        if (lane + 64 * i < L_act) l += __builtin_amdgcn_exp2f(sc[i] - mx);
    tail_rows([&](int, bool valid, float sv, float, float) { if (valid) l += __builtin_amdgcn_exp2f(sv - mx); }, L_act);
    l = wave_sum(l);
    const float inv = l > 0.f ? 1.0f / l : 0.f;
    _Float16 *wr = w + (int64_t)bh * Lp;
    // w is read (by the weighted row sum) up to the next multiple of 64 past the sequence's own rows, and must be
    // zero from L_act on; what lies beyond, up to the pitch, is never read
    const int fill = (L_act + 63) & ~63;                   // <= Lp
    float mu = 0.f;
#pragma unroll
    for (int i = 0; i < kKeep; ++i) {
        const int t = lane + 64 * i;
        if (t < fill) {
            _Float16 wt = (_Float16)0.f;
            if (t < L_act) {
                wt = (_Float16)(__builtin_amdgcn_exp2f(sc[i] - mx) * rs[i] * inv);
                mu = __builtin_fmaf((float)wt, mn[i], mu);
            }
            wr[t] = wt;
        }
    }
    tail_rows([&](int t, bool valid, float sv, float rstd, float mean) {
        if (t < fill) {
            _Float16 wt = (_Float16)0.f;
            if (valid) {
                wt = (_Float16)(__builtin_amdgcn_exp2f(sv - mx) * rstd * inv);
                mu = __builtin_fmaf((float)wt, mean, mu);
            }
            wr[t] = wt;
        }
    }, fill);
    mu = wave_sum(mu);
    if (lane == 0) sums[bh] = make_float4(mx, l, mu, 0.f);
}

// project: o_a[b,h,e] = W'_V[h dh + e, :] . Y[b,h,:] + b'_V for a slab of 32 output features of one head, then
// the join with the cached segment's (maximum, denominator, output).  Workgroup ids are regrouped so that the
// slabs of one head, which share that head's Y rows, run on one XCD.
template <int RB, int DT>
__global__ __launch_bounds__(256) void absorbed_project_kernel(const _Float16 *__restrict__ Wv, const _Float16 *__restrict__ Y,
                                                               const float *__restrict__ bv,
                                                               const float4 *__restrict__ sums,
                                                               const _Float16 *__restrict__ out_c, const float2 *__restrict__ lse_c,
                                                               _Float16 *__restrict__ out, int Bc, int H, int head_dim, int d)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    const int per_head = head_dim / skinny::kSlab;
    const int item = gemm::xcd_regroup(blockIdx.x, per_head * H);
    const int h = item / per_head;
    const int n0 = h * head_dim + (item % per_head) * skinny::kSlab;   // first V feature of the slab
    float (*red)[RB * 32][skinny::kSlab] = skinny::slab_product<RB, true, false, DT>(
        Wv + (int64_t)n0 * d, skinny::kSlab, d, Y + (int64_t)h * d, Bc, (int64_t)H * d, d, smem);
    for (int idx = tid; idx < Bc * skinny::kSlab; idx += 256) {
        const int b = idx / skinny::kSlab, c = idx % skinny::kSlab;
        const int n = n0 + c;
        const int64_t bh = (int64_t)b * H + h;
        const float4 sa = sums[bh];
        float o = (red[0][b][c] + red[1][b][c]) + (red[2][b][c] + red[3][b][c]);
        o += bv[n];
        // join of the two segments; a segment without tokens has denominator 0 and drops out, both empty: zero
        float m = sa.x, wc = 0.f, oc = 0.f;
        if (lse_c) {
            const float2 sc = lse_c[bh];
            m = fmaxf(sc.x, sa.x);
            wc = sc.y * __builtin_amdgcn_exp2f(sc.x - m);
            oc = skinny::stored_to_float<DT>(out_c + bh * head_dim + (n - h * head_dim));
        }
        const float wa = sa.y * __builtin_amdgcn_exp2f(sa.x - m);
        o = wc + wa > 0.f ? (wc * oc + wa * o) / (wc + wa) : 0.f;
        skinny::float_to_stored<DT>(out + bh * head_dim + (n - h * head_dim), o);
    }
}

// project, form for large layers: a workgroup per (head, part of the reduction axis) streams the head's rows of
// W'_V (head_dim <= 128 of them) once and shares the Y tile of the step through LDS (skinny::block_product),
// where the slab form above re-reads Y from L2 once per 32 features.  fp32 partial sums part[ks][b][n].
template <int RB, int DT>
__global__ __launch_bounds__(256) void absorbed_project_block_kernel(const _Float16 *__restrict__ Wv, const _Float16 *__restrict__ Y,
                                                                     float *__restrict__ part, int Bc, int H, int head_dim, int d,
                                                                     int steps_per_part)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int h = blockIdx.x, ks = blockIdx.y;
    const int steps = d / 64;
    const int k_begin = ks * steps_per_part;                               // < steps: the launcher leaves no part empty
    const int k_steps = steps - k_begin < steps_per_part ? steps - k_begin : steps_per_part;
    float16_t acc[RB];
    float m1[4], m2[4];
    _Float16 first[4];
    skinny::block_product<RB, true, false, DT>(Wv + (int64_t)h * head_dim * d, head_dim, d, Y + (int64_t)h * d, Bc, (int64_t)H * d,
                                           k_begin, k_steps, smem, acc, m1, m2, first);
    // acc[rb][r]: sequence 32 rb + 8 (r/4) + 4 (lane/32) + r%4, feature 32 wave + lane%32 of the head
    const int ln = lane & 31, lh = lane >> 5;
    const int c = 32 * wave + ln;
    if (c < head_dim) {
        float *dst = part + (int64_t)ks * Bc * d + h * head_dim + c;
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int m = 32 * rb + 8 * (r >> 2) + 4 * lh + (r & 3);
                if (m < Bc) dst[(int64_t)m * d] = acc[rb][r];
            }
    }
}

// Sum of the parts, bias, and the join with the cached segment (as in absorbed_project_kernel); 4 features per thread.
template <int DT>
__global__ __launch_bounds__(256) void absorbed_join_kernel(const float *__restrict__ part, int parts, const float *__restrict__ bv,
                                                            const float4 *__restrict__ sums,
                                                            const _Float16 *__restrict__ out_c, const float2 *__restrict__ lse_c,
                                                            _Float16 *__restrict__ out, int Bc, int H, int head_dim, int d)
{
    typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
    const int per_row = d / 4;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)Bc * per_row) return;
    const int b = (int)(idx / per_row), n = (int)(idx % per_row) * 4;     // 4 | head_dim: one head
    const int64_t stride = (int64_t)Bc * d;
    const float *src = part + (int64_t)b * d + n;
    float4_t o = *reinterpret_cast<const float4_t *>(src);
    for (int ks = 1; ks < parts; ++ks) o += *reinterpret_cast<const float4_t *>(src + ks * stride);
    const int h = n / head_dim;
    const int64_t bh = (int64_t)b * H + h;
    const float4 sa = sums[bh];
    float m = sa.x, wc = 0.f;
    half4_t oc = {0, 0, 0, 0};                             // 4 stored elements, whatever their type
    if (lse_c) {
        const float2 sc = lse_c[bh];
        m = fmaxf(sc.x, sa.x);
        wc = sc.y * __builtin_amdgcn_exp2f(sc.x - m);
        oc = *reinterpret_cast<const half4_t *>(out_c + (int64_t)b * d + n);
    }
    const float wa = sa.y * __builtin_amdgcn_exp2f(sa.x - m);
    half4_t res;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const float oa = o[j] + bv[n + j];
        const float ocj = skinny::stored_to_float<DT>(reinterpret_cast<const _Float16 *>(&oc) + j);
        skinny::float_to_stored<DT>(reinterpret_cast<_Float16 *>(&res) + j, wc + wa > 0.f ? (wc * ocj + wa * oa) / (wc + wa) : 0.f);
    }
    *reinterpret_cast<half4_t *>(out + (int64_t)b * d + n) = res;
}

// Below, the slab form of the projection is used (measured: 15.4 against 12.5 + 4.4 us at d = 4096, B = 32;
// 37 against 21 + 5 us at d = 5120, B = 64; 97 against 49 + 5 us at d = 9216, B = 64).
constexpr int kProjectBlockMinD = 5120;
constexpr int64_t kBlockModeMinRows = 128 * 512;           // from here on 128-row workgroups still fill the chip twice

template <int RB, int DT>
hipError_t launch_scores_as(const AbsorbedArgs &a, int Lp, hipStream_t s)
{
    const bool block_mode = (int64_t)a.B * a.L_act >= kBlockModeMinRows;
    const int per = block_mode ? 128 : skinny::kSlab;
    const int64_t items = (int64_t)((a.L_act + per - 1) / per) * a.B;
    if (items > 0x7fffffffLL) return hipErrorInvalidValue;
    auto kern = block_mode ? absorbed_scores_block_kernel<RB, DT> : absorbed_scores_kernel<RB, DT>;
    const int lds = block_mode ? skinny::block_lds_bytes<RB>() : skinny::lds_bytes<RB>() + skinny::kMomentBytes;
    static LdsOnce lds_once;
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kern), lds, lds_once);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)items), dim3(256), lds, s,
                       static_cast<const _Float16 *>(a.act), static_cast<const _Float16 *>(a.U), a.w_raw, a.stats,
                       a.B, a.L_act, Lp, a.H, a.d, a.eps);
    return hipGetLastError();
}

template <int RB>
hipError_t launch_scores(const AbsorbedArgs &a, int Lp, hipStream_t s)
{
    return a.dt == 1 ? launch_scores_as<RB, 1>(a, Lp, s) : launch_scores_as<RB, 0>(a, Lp, s);
}

template <int RB, int DT>
hipError_t launch_project_as(const AbsorbedArgs &a, int b0, int Bc, hipStream_t s)
{
    auto kern = absorbed_project_kernel<RB, DT>;
    constexpr int lds = skinny::lds_bytes<RB>();
    static LdsOnce lds_once;
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kern), lds, lds_once);
    if (e != hipSuccess) return e;
    const int64_t bh0 = (int64_t)b0 * a.H;
    hipLaunchKernelGGL(kern, dim3((unsigned)(a.head_dim / skinny::kSlab * a.H)), dim3(256), lds, s,
                       static_cast<const _Float16 *>(a.Wp) + (int64_t)a.d * a.d, static_cast<const _Float16 *>(a.Y) + bh0 * a.d,
                       a.bvec + a.d, a.sums + bh0,
                       a.L_kv > 0 ? static_cast<const _Float16 *>(a.out_c) + bh0 * a.head_dim : nullptr,
                       a.L_kv > 0 ? a.lse_c + bh0 : nullptr,
                       static_cast<_Float16 *>(a.out) + bh0 * a.head_dim, Bc, a.H, a.head_dim, a.d);
    return hipGetLastError();
}

template <int RB>
hipError_t launch_project(const AbsorbedArgs &a, int b0, int Bc, hipStream_t s)
{
    return a.dt == 1 ? launch_project_as<RB, 1>(a, b0, Bc, s) : launch_project_as<RB, 0>(a, b0, Bc, s);
}

template <int RB, int DT>
hipError_t launch_project_block_as(const AbsorbedArgs &a, int b0, int Bc, hipStream_t s)
{
    int parts, steps_per_part;
    absorbed_project_parts(a.d, a.H, &parts, &steps_per_part);
    if ((size_t)parts * Bc * a.d > a.proj_part_floats) return hipErrorInvalidValue;
    auto kern = absorbed_project_block_kernel<RB, DT>;
    constexpr int lds = skinny::block_lds_bytes<RB>();
    static LdsOnce lds_once;
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kern), lds, lds_once);
    if (e != hipSuccess) return e;
    const int64_t bh0 = (int64_t)b0 * a.H;
    hipLaunchKernelGGL(kern, dim3((unsigned)a.H, (unsigned)parts), dim3(256), lds, s,
                       static_cast<const _Float16 *>(a.Wp) + (int64_t)a.d * a.d, static_cast<const _Float16 *>(a.Y) + bh0 * a.d,
                       a.proj_part, Bc, a.H, a.head_dim, a.d, steps_per_part);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    const int64_t threads = (int64_t)Bc * (a.d / 4);
    hipLaunchKernelGGL(absorbed_join_kernel<DT>, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s,
                       a.proj_part, parts, a.bvec + a.d, a.sums + bh0,
                       a.L_kv > 0 ? static_cast<const _Float16 *>(a.out_c) + bh0 * a.head_dim : nullptr,
                       a.L_kv > 0 ? a.lse_c + bh0 : nullptr,
                       static_cast<_Float16 *>(a.out) + bh0 * a.head_dim, Bc, a.H, a.head_dim, a.d);
    return hipGetLastError();
}

template <int RB>
hipError_t launch_project_block(const AbsorbedArgs &a, int b0, int Bc, hipStream_t s)
{
    return a.dt == 1 ? launch_project_block_as<RB, 1>(a, b0, Bc, s) : launch_project_block_as<RB, 0>(a, b0, Bc, s);
}

}  // namespace

int absorbed_row_pitch(int L_act) { return (L_act + 63) / 64 * 64; }

// Parts of the reduction axis of the output projection: at most one workgroup per compute unit over the H heads
// (measured on d = 7168 and 9216: more parts cost more in partial sums than they gain), at least 4 steps of 64
// per part, no empty part.
void absorbed_project_parts(int d, int H, int *parts, int *steps_per_part)
{
    const int steps = d / 64;
    int want = 256 / (H > 0 ? H : 1);
    if (want > steps / 4) want = steps / 4;
    if (want < 1) want = 1;
    if (want > 8) want = 8;
    *steps_per_part = (steps + want - 1) / want;
    *parts = (steps + *steps_per_part - 1) / *steps_per_part;
}

namespace {

// What the steps of the checkpoint part need beyond AbsorbedArgs when the rows live in pool blocks.
struct PagedRows {
    const int32_t *blk_list;   // [B, list_pitch]: the checkpoint blocks of every request, in logical order
    const int32_t *n_rows;     // [B]: checkpoint rows of every request
    int list_pitch, blk_log2;
};

hipError_t launch_carry(const AbsorbedArgs &a, hipStream_t s)
{
    const int64_t d = a.d;
    // the queries through the key weights, at most kAbsorbMaxBatch sequences per launch
    for (int b0 = 0; b0 < a.B; b0 += kAbsorbMaxBatch) {
        const int Bc = a.B - b0 < kAbsorbMaxBatch ? a.B - b0 : kAbsorbMaxBatch;
        ColArgs c;
        c.S = static_cast<const _Float16 *>(a.Wp); c.s_batch = (int64_t)a.head_dim * d; c.ld_s = d; c.R = a.head_dim; c.n_cols = a.d;
        c.A = static_cast<const _Float16 *>(a.q) + b0 * d; c.a_batch = a.head_dim; c.ld_a = d; c.a_rows = Bc;
        c.Out = static_cast<_Float16 *>(a.U) + b0 * d; c.o_batch = a.B * d; c.ld_out = d;
        c.shift = nullptr; c.shift_batch = 0; c.shift_stride = 0;
        c.blk_list = nullptr; c.list_pitch = 0; c.blk_log2 = 0; c.R_list = nullptr;
        c.s_dt = a.dt; c.a_dt = a.dt;                      // prepared weights and queries as stored
        const hipError_t e = launch_column_product(c, a.H, s);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// softmax, weighted row sum, output projection and join; pr == nullptr: a.L_act contiguous rows per sequence
hipError_t launch_after_scores(const AbsorbedArgs &a, int Lp, const PagedRows *pr, hipStream_t s)
{
    const int64_t d = a.d;
    hipError_t e;
    const int64_t BH = (int64_t)a.B * a.H;
    hipLaunchKernelGGL(a.dt == 1 ? absorbed_softmax_kernel<1> : absorbed_softmax_kernel<0>, dim3((unsigned)((BH + 3) / 4)), dim3(256), 0, s,
                       static_cast<const _Float16 *>(a.q), a.w_raw, a.stats, a.cvec, a.bvec,
                       static_cast<_Float16 *>(a.w), a.sums, a.B, a.H, a.head_dim, a.L_act, Lp,
                       a.scale * 1.4426950408889634f, pr ? pr->n_rows : static_cast<const int32_t *>(nullptr),
                       pr ? Lp : a.L_act);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    {
        ColArgs c;
        c.S = static_cast<const _Float16 *>(a.act); c.s_batch = pr ? 0 : (int64_t)a.L_act * d; c.ld_s = d; c.R = a.L_act; c.n_cols = a.d;
        c.A = static_cast<const _Float16 *>(a.w); c.a_batch = (int64_t)a.H * Lp; c.ld_a = Lp; c.a_rows = a.H;
        c.Out = static_cast<_Float16 *>(a.Y); c.o_batch = a.H * d; c.ld_out = d;
        c.shift = &a.sums[0].z; c.shift_batch = 4 * (int64_t)a.H; c.shift_stride = 4;
        c.blk_list = pr ? pr->blk_list : nullptr; c.list_pitch = pr ? pr->list_pitch : 0; c.blk_log2 = pr ? pr->blk_log2 : 0;
        c.R_list = pr ? pr->n_rows : nullptr;
        c.s_dt = a.dt; c.a_dt = 0;                         // checkpoint rows as stored, weights w in fp16
        if ((e = launch_column_product(c, a.B, s)) != hipSuccess) return e;
    }
    for (int b0 = 0; b0 < a.B; b0 += kAbsorbMaxBatch) {
        const int Bc = a.B - b0 < kAbsorbMaxBatch ? a.B - b0 : kAbsorbMaxBatch;
        const bool block_mode = a.proj_part != nullptr && a.d >= kProjectBlockMinD;
        switch ((Bc + 31) / 32) {
        case 1: e = block_mode ? launch_project_block<1>(a, b0, Bc, s) : launch_project<1>(a, b0, Bc, s); break;
        case 2: e = block_mode ? launch_project_block<2>(a, b0, Bc, s) : launch_project<2>(a, b0, Bc, s); break;
        case 3: e = block_mode ? launch_project_block<3>(a, b0, Bc, s) : launch_project<3>(a, b0, Bc, s); break;
        default: e = block_mode ? launch_project_block<4>(a, b0, Bc, s) : launch_project<4>(a, b0, Bc, s); break;
        }
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// ---------------------------------------------------------------------------------------------------------
// Paged cache (Sec. 4.1, 4.2.1): the checkpoint rows of a request sit in blocks of the activation pool named by
// its row of the block table (entries < 0: checkpoint block ~entry).
//
// index: one wavefront per request walks its table row and leaves (a) the request's checkpoint blocks in logical
// order (list), their count, the rows of the last of them (only a request's final block can be partly filled) and
// the request's number of checkpoint rows; (b) the same view of its KV blocks: a table row that holds only them,
// in order, and the request's number of cached tokens, i.e. what the block-table attention kernel needs to walk
// the cached tokens alone.  Checkpoint blocks outside the pool prefix in use are left out.
__global__ __launch_bounds__(256) void paged_index_kernel(const int32_t *__restrict__ table, int max_blocks,
                                                          const int32_t *__restrict__ seq_len, int blk_log2, int n_act_used, int B,
                                                          int32_t *__restrict__ list, int32_t *__restrict__ count,
                                                          int32_t *__restrict__ last_rows, int32_t *__restrict__ n_rows,
                                                          int32_t *__restrict__ kv_table, int32_t *__restrict__ kv_len)
{
    const int lane = threadIdx.x & 63;
    const int b = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (b >= B) return;                                    // whole wavefront leaves together; no barrier in this kernel
    const int bt = 1 << blk_log2;
    const int len = seq_len[b];
    int nb = len > 0 ? (len + bt - 1) >> blk_log2 : 0;
    if (nb > max_blocks) nb = max_blocks;
    int k0 = 0, last_i = -1, c0 = 0, last_c = -1;
    for (int base = 0; base < nb; base += 64) {
        const int i = base + lane;
        const int32_t e = i < nb ? table[(int64_t)b * max_blocks + i] : 0;
        const bool is = i < nb && e < 0 && ~e < n_act_used;
        const bool kv = i < nb && e >= 0;
        const unsigned long long below = (1ull << lane) - 1ull;
        const unsigned long long mask = __ballot(is), cmask = __ballot(kv);
        if (is) list[(int64_t)b * max_blocks + k0 + __popcll(mask & below)] = ~e;
        if (kv) kv_table[(int64_t)b * max_blocks + c0 + __popcll(cmask & below)] = e;
        k0 += __popcll(mask);
        c0 += __popcll(cmask);
        if (mask) last_i = base + 63 - __builtin_clzll(mask);
        if (cmask) last_c = base + 63 - __builtin_clzll(cmask);
    }
    if (lane == 0) {
        auto rows_of = [&](int n_blocks, int last) {       // rows of n_blocks blocks whose last one is logical block `last`
            if (n_blocks <= 0) return 0;
            const int rest = len - (last << blk_log2);
            return ((n_blocks - 1) << blk_log2) + (rest < bt ? rest : bt);
        };
        count[b] = k0;
        n_rows[b] = rows_of(k0, last_i);
        last_rows[b] = k0 > 0 ? n_rows[b] - ((k0 - 1) << blk_log2) : bt;
        kv_len[b] = rows_of(c0, last_c);
    }
}

// cu[0] = 0, cu[b + 1] = cu[b] + len[b]: one wavefront, 64 requests per step.
__global__ __launch_bounds__(64) void paged_prefix_kernel(const int32_t *__restrict__ len, int B, int64_t *__restrict__ cu)
{
    const int lane = threadIdx.x;
    int64_t carry = 0;
    if (lane == 0) cu[0] = 0;
    for (int base = 0; base < B; base += 64) {
        const int i = base + lane;
        int64_t v = i < B ? len[i] : 0;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int64_t up = __shfl_up(v, off, 64);
            if (lane >= off) v += up;
        }
        if (i < B) cu[i + 1] = carry + v;
        carry += __shfl(v, 63, 64);
    }
}

// scores of 128 checkpoint rows of one request, as absorbed_scores_block_kernel (U is read once per 128 rows);
// rows are numbered inside the request in the order of its block list (raw, stats: pitch Lp per request) and
// found through that list (a block holds at least 16 rows, so the 8 rows of a load share a block).
template <int RB, int DT>
__global__ __launch_bounds__(256) void paged_scores_kernel(const _Float16 *__restrict__ act_pool, const _Float16 *__restrict__ U,
                                                           float *__restrict__ raw, float4 *__restrict__ stats,
                                                           const int32_t *__restrict__ list, const int32_t *__restrict__ n_rows,
                                                           int B, int max_blocks, int blk_log2, int groups, int Lp, int H, int d, float eps)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int item = gemm::xcd_regroup(blockIdx.x, groups * B);
    const int64_t b = item / groups;
    const int r0 = (item % groups) * 128;                  // first row of the workgroup inside the request
    const int total = n_rows[b];
    if (r0 >= total) return;                               // uniform over the workgroup, before any barrier
    const int n = total - r0 < 128 ? total - r0 : 128;
    const int32_t *blocks = list + b * max_blocks;
    const int mask = (1 << blk_log2) - 1;
    auto row_of = [=](int r) {
        const int rr = r0 + r;
        return act_pool + (((int64_t)blocks[rr >> blk_log2] << blk_log2) + (rr & mask)) * d;
    };
    float16_t acc[RB];
    float m1[4], m2[4];
    _Float16 first[4];
    skinny::block_product_rows<RB, false, true, DT>(row_of, n, U + b * d, H, (int64_t)B * d, 0, d / 64, smem, acc, m1, m2, first);
    const int rw = r0 + 32 * wave;                         // first row of this wavefront
    const int rows = total - rw < 32 ? (total - rw > 0 ? total - rw : 0) : 32;
    const int ln = lane & 31, lh = lane >> 5;
    if (ln < rows) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int h = 32 * rb + 8 * (r >> 2) + 4 * lh + (r & 3);
                if (h < H) raw[(b * H + h) * Lp + rw + ln] = acc[rb][r];
            }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int row = 8 * j + (lane >> 3);
        if ((lane & 7) == 0 && row < rows) stats[b * Lp + rw + row] = row_stats(m1[j], m2[j], (float)first[j], d, eps);
    }
}

template <int RB, int DT>
hipError_t launch_paged_scores_as(const PagedAbsorbedArgs &p, int Lp, int blk_log2, hipStream_t s)
{
    const AbsorbedArgs &a = p.abs;
    const int groups = (a.L_act + 127) / 128;              // of the longest request possible; shorter ones leave early
    const int64_t items = (int64_t)a.B * groups;
    if (items <= 0) return hipSuccess;
    if (items > 0x7fffffffLL) return hipErrorInvalidValue;
    auto kern = paged_scores_kernel<RB, DT>;
    constexpr int lds = skinny::block_lds_bytes<RB>();
    static LdsOnce lds_once;
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kern), lds, lds_once);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)items), dim3(256), lds, s,
                       static_cast<const _Float16 *>(a.act), static_cast<const _Float16 *>(a.U), a.w_raw, a.stats,
                       p.list, p.n_rows, a.B, p.max_blocks, blk_log2, groups, Lp, a.H, a.d, a.eps);
    return hipGetLastError();
}

template <int RB>
hipError_t launch_paged_scores(const PagedAbsorbedArgs &p, int Lp, int blk_log2, hipStream_t s)
{
    return p.abs.dt == 1 ? launch_paged_scores_as<RB, 1>(p, Lp, blk_log2, s) : launch_paged_scores_as<RB, 0>(p, Lp, blk_log2, s);
}

}  // namespace

hipError_t launch_absorbed(const AbsorbedArgs &a, hipStream_t s)
{
    if (a.B <= 0 || a.L_act <= 0) return hipSuccess;
    if (a.H > kAbsorbMaxHeads || a.d % 64 != 0 || a.B > 65535 || (int64_t)a.H * a.head_dim != a.d || (a.dt != 0 && a.dt != 1))
        return hipErrorInvalidValue;
    const int Lp = absorbed_row_pitch(a.L_act);
    hipError_t e = launch_carry(a, s);
    if (e != hipSuccess) return e;
    switch ((a.H + 31) / 32) {
    case 1: e = launch_scores<1>(a, Lp, s); break;
    case 2: e = launch_scores<2>(a, Lp, s); break;
    case 3: e = launch_scores<3>(a, Lp, s); break;
    default: e = launch_scores<4>(a, Lp, s); break;
    }
    if (e != hipSuccess) return e;
    return launch_after_scores(a, Lp, nullptr, s);
}

// The two views of the block table that the paged step without regeneration works on (see paged_index_kernel).
hipError_t launch_paged_index(const PagedAbsorbedArgs &p, hipStream_t s)
{
    const AbsorbedArgs &a = p.abs;
    if (a.B <= 0) return hipSuccess;
    if (p.block_tokens < 16 || (p.block_tokens & (p.block_tokens - 1)) != 0 || p.max_blocks <= 0) return hipErrorInvalidValue;
    int blk_log2 = 0;
    while ((1 << blk_log2) < p.block_tokens) ++blk_log2;
    hipLaunchKernelGGL(paged_index_kernel, dim3((unsigned)((a.B + 3) / 4)), dim3(256), 0, s,
                       p.block_table, p.max_blocks, p.seq_len, blk_log2, p.n_act_used, a.B, p.list, p.count, p.last_rows, p.n_rows,
                       p.kv_table, p.kv_len);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(paged_prefix_kernel, dim3(1), dim3(64), 0, s, p.kv_len, a.B, p.kv_cu);
    return hipGetLastError();
}

// After launch_paged_index (and the attention over the KV view).  a.abs: act = the activation pool, L_act =
// max_blocks * block_tokens (the most rows a request can have), L_kv != 0 iff out_c / lse_c hold the attention
// over the KV blocks; stats and w_raw, w have pitch absorbed_row_pitch(L_act).
hipError_t launch_paged_absorbed(const PagedAbsorbedArgs &p, hipStream_t s)
{
    const AbsorbedArgs &a = p.abs;
    if (a.B <= 0) return hipSuccess;
    if (a.H > kAbsorbMaxHeads || a.d % 64 != 0 || a.B > 65535 || (int64_t)a.H * a.head_dim != a.d || (a.dt != 0 && a.dt != 1))
        return hipErrorInvalidValue;
    if (p.block_tokens < 16 || (p.block_tokens & (p.block_tokens - 1)) != 0 || p.max_blocks <= 0 || a.L_act != p.max_blocks * p.block_tokens)
        return hipErrorInvalidValue;
    int blk_log2 = 0;
    while ((1 << blk_log2) < p.block_tokens) ++blk_log2;
    const int Lp = absorbed_row_pitch(a.L_act);
    hipError_t e = launch_carry(a, s);
    if (e != hipSuccess) return e;
    switch ((a.H + 31) / 32) {
    case 1: e = launch_paged_scores<1>(p, Lp, blk_log2, s); break;
    case 2: e = launch_paged_scores<2>(p, Lp, blk_log2, s); break;
    case 3: e = launch_paged_scores<3>(p, Lp, blk_log2, s); break;
    default: e = launch_paged_scores<4>(p, Lp, blk_log2, s); break;
    }
    if (e != hipSuccess) return e;
    PagedRows pr;
    pr.blk_list = p.list; pr.n_rows = p.n_rows; pr.list_pitch = p.max_blocks; pr.blk_log2 = blk_log2;
    return launch_after_scores(a, Lp, &pr, s);
}

}  // namespace hk
