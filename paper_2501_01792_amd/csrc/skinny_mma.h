// Product of one slab of 32 rows streamed from HBM with a small set of rows kept hot in L2, on the matrix
// cores: D[m][c] = sum_k A[m][k] * S[c][k], m < 32 RB small rows, c < 32 streamed rows, k < d.
// Shared by the kernels whose cost is one pass over a large row-major operand and whose other operand
// has few rows (current-token QKV generation; the weight-absorbed decode).
//
// One workgroup of 4 wavefronts per slab.  Each wavefront takes a quarter of the reduction axis, streams
// its part of the slab straight into registers with whole-line loads (8 lanes per 128-byte line, several
// steps in flight), turns it into MFMA operand layout through a private 4 KiB LDS block and multiplies
// it with the matching part of the small operand (fetched the same way, through L2).  The four partial
// sums are left in LDS for the caller's epilogue.  On request the pass also leaves the first two moments of
// every streamed row (shifted by the row's first element), which is what a LayerNorm of those rows needs.
//
// block_product is the form for many streamed rows: 128 per workgroup, 32 per wavefront, every wavefront
// walking the same range of the reduction axis, the small operand's tile shared through LDS.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "elem.h"

namespace hk {
namespace skinny {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef float float16_t __attribute__((ext_vector_type(16)));

// The kernels built on these products compute in fp16 whatever the storage type of the tensors: an operand stored as
// bfloat16 (SDT = 1) is converted piece by piece on its way from the load to LDS.  The conversion is exact for
// magnitudes in fp16's normal range (a bfloat16 has 8 significant bits, an fp16 11); larger magnitudes stop at
// 65504, and below 2^-14 the low bits are dropped.  Pointers to such operands are passed as _Float16 pointers
// (same size and addressing).
typedef unsigned uint4v_t __attribute__((ext_vector_type(4)));
template <int SDT>
__device__ __forceinline__ half8_t to_half8(half8_t raw)
{
    if constexpr (SDT == 0) {
        return raw;
    } else {
        const uint4v_t u = __builtin_bit_cast(uint4v_t, raw);
        uint4v_t o;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float lo = __builtin_bit_cast(float, u[e] << 16), hi = __builtin_bit_cast(float, u[e] & 0xffff0000u);
            o[e] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pkrtz(lo, hi));
        }
        return __builtin_bit_cast(half8_t, o);
    }
}
// One stored element as fp32, and fp32 to one stored element (round to nearest even).
template <int SDT>
__device__ __forceinline__ float stored_to_float(const _Float16 *p)
{
    if constexpr (SDT == 0) return (float)*p;
    else return __builtin_bit_cast(float, (unsigned)*reinterpret_cast<const unsigned short *>(p) << 16);
}
template <int SDT>
__device__ __forceinline__ void float_to_stored(_Float16 *p, float v)
{
    if constexpr (SDT == 0) *p = (_Float16)v;
    else *reinterpret_cast<__bf16 *>(p) = (__bf16)v;
}
// One stored element as fp16 (same rule as to_half8).
template <int SDT>
__device__ __forceinline__ _Float16 stored_to_half(const _Float16 *p)
{
    if constexpr (SDT == 0) return *p;
    else {
        const unsigned pk = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_pkrtz(stored_to_float<1>(p), 0.f));
        return __builtin_bit_cast(_Float16, (unsigned short)(pk & 0xffffu));
    }
}

constexpr int kSlab = 32;                // streamed rows per workgroup
constexpr int kStepK = 64;               // reduction elements per step of one wavefront
constexpr int kBlockBytes = 32 * kStepK * 2;               // 4 KiB: 32 rows x 128 bytes of one operand, one step

// Bytes of dynamic LDS of one workgroup: per wavefront one 4 KiB block for the streamed operand and RB for
// the small one while the loop runs; afterwards the same memory holds the four partial sums.
template <int RB>
constexpr int lds_bytes()
{
    return 4 * (1 + RB) * kBlockBytes > 4 * RB * 32 * kSlab * 4 ? 4 * (1 + RB) * kBlockBytes : 4 * RB * 32 * kSlab * 4;
}

// Shifted rows and their moments (STATS): every streamed row enters the product minus its first element,
// D[m][c] = sum_k A[m][k] (S[c][k] - S[c][0]), and after the call, for wavefront w and slab row c,
//   moments(smem)[w][c] = (sum_k (S[c][k] - S[c][0]), sum_k (S[c][k] - S[c][0])^2) over k quarter w
// (differences taken in fp16, |difference| < 65504 assumed; sums in fp32).  The shift keeps a row mean that
// is large against the row's spread out of the variance and out of the product.  The moments live behind the
// partial sums: add kMomentBytes to the LDS size.
constexpr int kMomentBytes = 4 * kSlab * 2 * 4;
template <int RB>
__device__ __forceinline__ float (*moments(unsigned char *smem))[kSlab][2]
{
    return reinterpret_cast<float (*)[kSlab][2]>(smem + lds_bytes<RB>());
}

// S: first row of the slab (row stride ld_s elements; rows >= s_rows are not read: the last valid row stands
// in for them), stored as SDT.  A: first small row (row stride ld_a; rows >= a_rows likewise), fp16.  d % 64 == 0.
// Returns red with red[w][m][c], w = 0..3, the partial sum of k quarter w; a barrier has been passed.
template <int RB, bool NT, bool STATS = false, int SDT = 0>
__device__ __forceinline__ float (*slab_product(const _Float16 *__restrict__ S, int s_rows, int64_t ld_s,
                                                const _Float16 *__restrict__ A, int a_rows, int64_t ld_a,
                                                int d, unsigned char *smem))[RB * 32][kSlab]
{
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // this wavefront's quarter of the reduction axis, in steps of 64 (the last quarter takes the remainder)
    const int steps_total = d / kStepK;
    const int per = (steps_total + 3) / 4;
    const int s_begin = wave * per < steps_total ? wave * per : steps_total;
    const int s_end = s_begin + per < steps_total ? s_begin + per : steps_total;

    // Global side: one load instruction covers 8 rows x 128 bytes, 8 lanes per row (whole lines; two lanes
    // per row, which is what the MFMA operand layout would ask for, leaves the L2 with four 16-byte
    // requests per line and runs at a quarter of the rate).  Lane l of load j: row 8 j + l / 8, chunk l % 8.
    const int g_row = lane >> 3, g_chunk = lane & 7;
    const _Float16 *wp[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        int c = 8 * j + g_row;
        if (c >= s_rows) c = s_rows - 1;                   // clamp: rows past the end are computed, never used
        wp[j] = S + (int64_t)c * ld_s + 8 * g_chunk;
    }
    const _Float16 *xp[RB][4];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int m = rb * 32 + 8 * j + g_row;
            if (m >= a_rows) m = a_rows - 1;               // clamp: rows past the end are computed, never used
            xp[rb][j] = A + (int64_t)m * ld_a + 8 * g_chunk;
        }
    // LDS side (private to the wavefront, so no barrier): a block is 32 rows of 128 bytes, the 16-byte chunk
    // index XOR-ed with (row / 2) % 8, which makes both the row-wise writes and the MFMA-operand reads
    // (32 rows x one chunk per half wavefront) conflict-free.
    unsigned char *my = smem + wave * (1 + RB) * kBlockBytes;
    int wr_off[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int row = 8 * j + g_row;
        wr_off[j] = row * 128 + ((g_chunk ^ ((row >> 1) & 7)) << 4);
    }
    const int ln = lane & 31, lh = lane >> 5;              // operand row inside a block, k half of an MFMA
    int rd_off[4];
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) rd_off[jj] = ln * 128 + (((2 * jj + lh) ^ ((ln >> 1) & 7)) << 4);

    float16_t acc[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[rb][r] = 0.f;

    // row moments: lane (g_row, g_chunk) sums its 8-element pieces of rows 8 j + g_row
    float m1[4] = {0.f, 0.f, 0.f, 0.f}, m2[4] = {0.f, 0.f, 0.f, 0.f};
    half8_t shift[4];
    if constexpr (STATS) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const _Float16 c = stored_to_half<SDT>(wp[j] - 8 * g_chunk);   // first element of the row
            shift[j] = half8_t{c, c, c, c, c, c, c, c};
        }
    }

    // Streamed pieces are fetched kDepth - 1 steps ahead, small-operand pieces kXDepth - 1 steps ahead.  Vector memory
    // loads complete in issue order as far as s_waitcnt can tell, so inside a step the small-operand loads (L2) are
    // issued BEFORE the streamed loads (HBM): the wait for the former then leaves the latter in flight.
    constexpr int kDepth = RB <= 2 ? 6 : 4;
    constexpr int kXDepth = RB <= 2 ? 3 : 2;               // divides kDepth
    half8_t wv[kDepth][4];
    half8_t xv[kXDepth][RB][4];
    auto load_w = [&](int slot, int sc) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
        {
            const half8_t *src = reinterpret_cast<const half8_t *>(wp[j] + (int64_t)sc * kStepK);
            wv[slot][j] = NT ? __builtin_nontemporal_load(src) : *src;
        }
    };
    auto load_x = [&](int slot, int sc) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                xv[slot][rb][j] = *reinterpret_cast<const half8_t *>(xp[rb][j] + (int64_t)sc * kStepK);
    };
    // Every load of the loop is unconditional (steps past the end re-read the last step, an L2 hit), so
    // that the number of loads in flight at each wait is a compile-time fact; only the MFMAs are guarded.
    const int last = s_end - 1;
    auto clamp = [&](int sc) { return sc < last ? sc : last; };
    if (s_begin < s_end) {
#pragma unroll
        for (int u = 0; u < kXDepth - 1; ++u) load_x(u, clamp(s_begin + u));
#pragma unroll
        for (int u = 0; u < kDepth - 1; ++u) load_w(u, clamp(s_begin + u));
        for (int s = s_begin; s < s_end; s += kDepth) {
#pragma unroll
            for (int u = 0; u < kDepth; ++u) {             // unrolled so that every register slot index is static
                const int sc = s + u;
                load_x((u + kXDepth - 1) % kXDepth, clamp(sc + kXDepth - 1));
                load_w((u + kDepth - 1) % kDepth, clamp(sc + kDepth - 1));
                if (sc < s_end) {
                    // registers (row-wise) -> LDS -> registers (MFMA operand layout)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        half8_t piece = to_half8<SDT>(wv[u][j]);
                        if constexpr (STATS) {
                            piece -= shift[j];             // the product is taken with the shifted rows
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const half2_t pr = {piece[2 * e], piece[2 * e + 1]};
                                m1[j] = __builtin_amdgcn_fdot2(pr, half2_t{(_Float16)1.f, (_Float16)1.f}, m1[j], false);
                                m2[j] = __builtin_amdgcn_fdot2(pr, pr, m2[j], false);
                            }
                        }
                        *reinterpret_cast<half8_t *>(my + wr_off[j]) = piece;
                    }
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            *reinterpret_cast<half8_t *>(my + (1 + rb) * kBlockBytes + wr_off[j]) = xv[u % kXDepth][rb][j];
                    half8_t wf[4];
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj) wf[jj] = *reinterpret_cast<const half8_t *>(my + rd_off[jj]);
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
                        for (int jj = 0; jj < 4; ++jj) {
                            const half8_t xf = *reinterpret_cast<const half8_t *>(my + (1 + rb) * kBlockBytes + rd_off[jj]);
                            acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(xf, wf[jj], acc[rb], 0, 0, 0);
                        }
                }
            }
        }
    }

    if constexpr (STATS) {
        float (*mom)[kSlab][2] = moments<RB>(smem);        // behind everything else in LDS: no aliasing
#pragma unroll
        for (int j = 0; j < 4; ++j) {
#pragma unroll
            for (int off = 1; off < 8; off <<= 1) {
                m1[j] += __shfl_xor(m1[j], off, 64);
                m2[j] += __shfl_xor(m2[j], off, 64);
            }
            if (g_chunk == 0) {
                mom[wave][8 * j + g_row][0] = m1[j];
                mom[wave][8 * j + g_row][1] = m2[j];
            }
        }
    }

    // ---- the four k quarters meet in LDS (the staging blocks are dead once every wavefront is here).
    // acc[rb][r]: small row 32 rb + 8 (r/4) + 4 (lane/32) + r%4, streamed row lane%32
    __syncthreads();
    float (*red)[RB * 32][kSlab] = reinterpret_cast<float (*)[RB * 32][kSlab]>(smem);
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            red[wave][rb * 32 + 8 * (r >> 2) + 4 * lh + (r & 3)][ln] = acc[rb][r];
    __syncthreads();

    return red;
}

// ---------------------------------------------------------------------------------------------------------
// block_product: D[m][c] = sum_k A[m][k] * S[c][k] over k in [64 k_begin, 64 (k_begin + k_steps)), for the 32
// streamed rows c = 32 wave + lane % 32 of a block of up to 128 rows that the 4 wavefronts of a workgroup share.
//
// The tile of the small operand of a step (32 RB rows x 128 bytes) is the same for the four wavefronts: it is
// fetched once per workgroup with whole-line loads (as far ahead as the streamed rows, because vector memory
// loads retire in issue order) and shared through a double-buffered LDS tile, one barrier per step; so the
// small operand is read once per 128 streamed rows.  The streamed rows go from HBM to registers to the
// wavefront's private LDS block (row-wise in, MFMA operand layout out) as in slab_product.  There is no
// reduction across wavefronts: the result stays in registers,
//   acc[rb][r] = D[32 rb + 8 (r/4) + 4 (lane/32) + r%4][32 wave + lane%32].
// STATS: rows enter the product minus their first element; m1[j], m2[j] are the first two moments of row
// 32 wave + 8 j + lane / 8 (complete in every lane of the row's 8), first[j] that row's first element.
// All 256 threads must call it (barriers), with the same k range.  n_rows >= 1 rows of S are valid; rows
// past them are computed from the last valid row and must not be stored.
template <int RB>
constexpr int block_lds_bytes() { return 4 * kBlockBytes + 2 * RB * kBlockBytes; }

// row_of(r) is the address of streamed row r, r < n_rows (rows need not be evenly spaced: they may sit in
// blocks scattered over a pool).
// SDT: storage type of the streamed rows (the small operand A is fp16).
template <int RB, bool NT, bool STATS, int SDT = 0, typename RowOf>
__device__ __forceinline__ void block_product_rows(RowOf row_of, int n_rows,
                                                   const _Float16 *__restrict__ A, int a_rows, int64_t ld_a,
                                                   int k_begin, int k_steps, unsigned char *smem,
                                                   float16_t (&acc)[RB], float (&m1)[4], float (&m2)[4], _Float16 (&first)[4])
{
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g_row = lane >> 3, g_chunk = lane & 7;
    const int ln = lane & 31, lh = lane >> 5;
    const _Float16 *sp[4];
    half2_t shift[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        int r = 32 * wave + 8 * j + g_row;
        if (r >= n_rows) r = n_rows - 1;
        const _Float16 *row = row_of(r);
        if constexpr (STATS) {
            first[j] = stored_to_half<SDT>(row);
            shift[j] = half2_t{first[j], first[j]};
        } else {
            first[j] = (_Float16)0.f;
        }
        sp[j] = row + 64 * (int64_t)k_begin + 8 * g_chunk;
        m1[j] = 0.f;
        m2[j] = 0.f;
    }
    const int t_row = tid >> 3, t_chunk = tid & 7;         // the shared tile: thread -> (row of every 32-row block, chunk)
    const _Float16 *ap[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        int m = rb * 32 + t_row;
        if (m >= a_rows) m = a_rows - 1;
        ap[rb] = A + (int64_t)m * ld_a + 64 * (int64_t)k_begin + 8 * t_chunk;
    }
    // LDS blocks: 32 rows of 128 bytes, chunk index XOR-ed with (row / 2) % 8
    int wr_off[4], rd_off[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int row = 8 * j + g_row;
        wr_off[j] = row * 128 + ((g_chunk ^ ((row >> 1) & 7)) << 4);
        rd_off[j] = ln * 128 + (((2 * j + lh) ^ ((ln >> 1) & 7)) << 4);
    }
    const int t_wr = t_row * 128 + ((t_chunk ^ ((t_row >> 1) & 7)) << 4);
    unsigned char *my = smem + wave * kBlockBytes;
    unsigned char *tile = smem + 4 * kBlockBytes;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[rb][r] = 0.f;

    constexpr int kDepth = RB <= 1 ? 6 : 5;
    half8_t sv[kDepth][4];
    half8_t av[kDepth][RB];
    const int last = k_steps - 1;
    auto fetch = [&](int slot, int sc) {                   // the small operand (L2) before the streamed rows (HBM)
        if (sc > last) sc = last;
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) av[slot][rb] = *reinterpret_cast<const half8_t *>(ap[rb] + 64 * sc);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const half8_t *src = reinterpret_cast<const half8_t *>(sp[j] + 64 * sc);
            sv[slot][j] = NT ? __builtin_nontemporal_load(src) : *src;
        }
    };
    auto put_a = [&](int slot, int buf) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
            *reinterpret_cast<half8_t *>(tile + (buf * RB + rb) * kBlockBytes + t_wr) = av[slot][rb];
    };
    if (k_steps <= 0) return;                              // uniform over the workgroup
#pragma unroll
    for (int u = 0; u < kDepth - 1; ++u) fetch(u, u);
    put_a(0, 0);
    __syncthreads();
    for (int s = 0; s < k_steps; s += kDepth) {
#pragma unroll
        for (int u = 0; u < kDepth; ++u) {
            const int sc = s + u;
            fetch((u + kDepth - 1) % kDepth, sc + kDepth - 1);
            if (sc < k_steps) {                            // uniform over the workgroup
                put_a((u + 1) % kDepth, (sc + 1) & 1);     // the tile of step sc + 1, for the next pass
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    half8_t piece = to_half8<SDT>(sv[u][j]);
                    if constexpr (STATS) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const half2_t pr = half2_t{piece[2 * e], piece[2 * e + 1]} - shift[j];
                            m1[j] = __builtin_amdgcn_fdot2(pr, half2_t{(_Float16)1.f, (_Float16)1.f}, m1[j], false);
                            m2[j] = __builtin_amdgcn_fdot2(pr, pr, m2[j], false);
                            piece[2 * e] = pr[0];
                            piece[2 * e + 1] = pr[1];
                        }
                    }
                    *reinterpret_cast<half8_t *>(my + wr_off[j]) = piece;
                }
                // The operand fragments of k piece jj + 1 are read while the MFMAs of piece jj run: left to the
                // compiler every MFMA waits for its own LDS read (register pressure makes it reuse one register set).
                half8_t wf[2], af[2][RB];
                auto read_piece = [&](int jj) {
                    wf[jj & 1] = *reinterpret_cast<const half8_t *>(my + rd_off[jj]);
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb)
                        af[jj & 1][rb] = *reinterpret_cast<const half8_t *>(tile + ((sc & 1) * RB + rb) * kBlockBytes + rd_off[jj]);
                };
                read_piece(0);
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) {
                    if (jj + 1 < 4) read_piece(jj + 1);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb)
                        acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[jj & 1][rb], wf[jj & 1], acc[rb], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                }
                __syncthreads();                           // tile sc + 1 is complete; tile sc is free for sc + 2
            }
        }
    }
    if constexpr (STATS) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int off = 1; off < 8; off <<= 1) {
                m1[j] += __shfl_xor(m1[j], off, 64);
                m2[j] += __shfl_xor(m2[j], off, 64);
            }
    }
}

// Evenly spaced rows: S is the first row of the block, ld_s the distance between rows.
template <int RB, bool NT, bool STATS, int SDT = 0>
__device__ __forceinline__ void block_product(const _Float16 *__restrict__ S, int n_rows, int64_t ld_s,
                                              const _Float16 *__restrict__ A, int a_rows, int64_t ld_a,
                                              int k_begin, int k_steps, unsigned char *smem,
                                              float16_t (&acc)[RB], float (&m1)[4], float (&m2)[4], _Float16 (&first)[4])
{
    block_product_rows<RB, NT, STATS, SDT>([=](int r) { return S + (int64_t)r * ld_s; }, n_rows, A, a_rows, ld_a, k_begin, k_steps,
                                      smem, acc, m1, m2, first);
}

}  // namespace skinny
}  // namespace hk
