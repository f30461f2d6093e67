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
// bytes): an HBM streaming kernel, one launch (qkv_fused_kernel below).
#include "hk_internal.h"
#include "elem.h"
#include "skinny_mma.h"

namespace hk {
namespace {

using skinny::float16_t;

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));

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

// Everything in one launch.  A workgroup owns 32 NW output features (rows of Wq, or of [Wk; Wv]); its wavefronts form
// KS groups of NW, every group takes a contiguous part of the reduction axis (the problem has too few output
// features to fill the chip with wavefronts that each walk the whole axis, and the bytes in flight per wavefront
// are bounded by its registers), and the groups' partial results meet in LDS at the end.  Each wavefront streams
// its 32 weight rows from HBM with whole-line loads, several steps of 64 reduction elements in flight, through a
// private LDS block into MFMA operand layout (v_mfma_f32_32x32x16).  The other operand is built on the fly, once
// per group and step, into a double-buffered LDS tile shared by the group's wavefronts.  The LayerNorm is folded
// around the product so that the tile needs nothing but the raw input rows:
//     out[m][n] = rstd_m * S[m][n] + rstd_m (s_m - mean_m) * G[n] + T[n] + bias[n],
//     S[m][n] = sum_k a[m][k] W[n][k],  a[m][k] = round(round(x[m][k] - s_m) * gamma[k]),
//     G[n] = sum_k gamma[k] W[n][k],    T[n] = sum_k beta[k] W[n][k],
// where s_m is a shift near the row's mean (the mean of its first 64 elements) that keeps a large common offset
// of a row out of the rounded operand.  G and T are summed beside the MFMAs from the weight pieces a lane holds
// anyway (v_dot2 with the matching pieces of gamma and beta, fp32), and the row moments (sum and sum of squares of
// the rounded x - s_m, fp32) from the chunks the threads load for the tile.  The epilogue (the first group) adds
// the groups' parts, applies the statistics, adds the bias, rounds and stores q, or the K / V row of the token
// (contiguous cache, or the block its table entry names).  Workgroup 0 also copies the raw input rows into the
// checkpoint store when asked.
struct FusedArgs {
    const void *x, *gamma, *beta, *Wq, *Wkv, *bq, *bkv;
    void *q_out, *K_dst, *V_dst, *act_dst;
    int64_t act_row_stride;
    int B, d, n_heads, head_dim, L_cap, tok_pos, q_blocks;
    float eps;
    PagedDst pd;
};

template <int RB, int NW, int KS>
constexpr int fused_lds_bytes()
{
    // the loop: a private block per wavefront, a double-buffered tile per group; afterwards the same memory holds the
    // groups' partial accumulators; behind it the small tables of the epilogue
    constexpr int loop = NW * KS * skinny::kBlockBytes + KS * 2 * RB * skinny::kBlockBytes;
    constexpr int red = KS * NW * RB * 16 * 64 * 4;
    constexpr int tables = KS * RB * 32 * 8 /* moments */ + KS * 2 * 32 * NW * 4 /* G, T */ + RB * 32 * 8 /* statistics */ + RB * 32 * 8 /* row destinations */;
    return (loop > red ? loop : red) + tables;
}

template <int RB, int NW, int KS, int kDepth, int DT>
__global__ __launch_bounds__(64 * NW * KS) void qkv_fused_kernel(FusedArgs p)
{
    typedef typename Elem<DT>::T elem_t;
    typedef typename Elem<DT>::V8 vec8_t;
    typedef typename Elem<DT>::V2 vec2_t;
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int GT = 64 * NW;                  // threads of a group
    constexpr int NF = 32 * NW;                  // output features of the workgroup
    constexpr int RPP = 8 * NW;                  // tile rows one pass of a group covers
    constexpr int P = 32 * RB / RPP;             // passes per tile
    constexpr int KB = skinny::kBlockBytes;
    constexpr int kLoop = NW * KS * KB + KS * 2 * RB * KB;
    constexpr int kRed = KS * NW * RB * 16 * 64 * 4;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = wave / NW, wg = wave % NW;   // group (part of the reduction axis), wavefront inside the group
    const int gtid = tid - grp * GT;             // thread inside the group
    const int B = p.B, d = p.d;
    const int k_steps = d / 64;
    const int steps_g = (k_steps + KS - 1) / KS;                            // steps of a group (the last ones may have fewer)
    const int k_begin = grp * steps_g;
    const int my_steps = k_steps - k_begin < steps_g ? (k_steps - k_begin > 0 ? k_steps - k_begin : 0) : steps_g;
    const bool is_q = (int)blockIdx.x < p.q_blocks;
    const int n0 = (is_q ? (int)blockIdx.x : (int)blockIdx.x - p.q_blocks) * (32 * NW);   // first row inside its weight array
    const int n_total = is_q ? d : 2 * d;
    const int n_rows = n_total - n0 < 32 * NW ? n_total - n0 : 32 * NW;
    const elem_t *W = static_cast<const elem_t *>(is_q ? p.Wq : p.Wkv) + (int64_t)n0 * d;
    const elem_t *x = static_cast<const elem_t *>(p.x);
    const elem_t *gamma = static_cast<const elem_t *>(p.gamma), *beta = static_cast<const elem_t *>(p.beta);

    unsigned char *my = smem + wave * KB;                                   // this wavefront's private block
    unsigned char *tile = smem + NW * KS * KB + grp * 2 * RB * KB;          // this group's [2][RB] blocks of 32 rows x 128 bytes
    float *red = reinterpret_cast<float *>(smem);                           // after the loop: [KS][NW][RB * 16][64]
    unsigned char *tab = smem + (kLoop > kRed ? kLoop : kRed);
    float2 *mom = reinterpret_cast<float2 *>(tab);                          // [KS][32 RB]: a group's row moments
    float *gt = reinterpret_cast<float *>(mom + KS * RB * 32);              // [KS][2][NF]: a group's parts of G, T
    float2 *stats = reinterpret_cast<float2 *>(gt + KS * 2 * NF);           // [32 RB]: (rstd, (shift - mean) rstd)
    int64_t *rowdst = reinterpret_cast<int64_t *>(stats + RB * 32);         // [32 RB]: where row m's K/V row starts, or -1

    // ---- streamed side: lane (g_row, g_chunk) of load j fetches chunk g_chunk of weight row 32 wg + 8 j + g_row
    const int g_row = lane >> 3, g_chunk = lane & 7;
    const int ln = lane & 31, lh = lane >> 5;
    const elem_t *sp[4];
    int wr_off[4], rd_off[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        int r = 32 * wg + 8 * j + g_row;
        if (r >= n_rows) r = n_rows - 1;                                    // rows past the end: computed, never stored
        sp[j] = W + (int64_t)r * d + 64 * (int64_t)k_begin + 8 * g_chunk;
        const int row = 8 * j + g_row;
        wr_off[j] = row * 128 + ((g_chunk ^ ((row >> 1) & 7)) << 4);
        rd_off[j] = ln * 128 + (((2 * j + lh) ^ ((ln >> 1) & 7)) << 4);
    }
    // ---- tile side: thread (t_row, t_chunk) of pass q builds chunk t_chunk of tile row q RPP + t_row.
    // Tile rows: 0 .. B-1 the input rows, the rest zero.  t_chunk == g_chunk: the pieces of gamma and beta a thread
    // fetches for the tile are also the ones that match its pieces of the weight rows.
    const int t_row = gtid >> 3, t_chunk = gtid & 7;
    const elem_t *rp[P];
    bool is_row[P];
    int t_wr[P];
#pragma unroll
    for (int q = 0; q < P; ++q) {
        const int m = q * RPP + t_row;
        is_row[q] = m < B;
        rp[q] = x + (int64_t)(m < B ? m : B - 1) * d + 8 * t_chunk;         // padding rows: a valid address, zeros in the tile
        const int rb = m >> 5, row = m & 31;
        t_wr[q] = rb * KB + row * 128 + ((t_chunk ^ ((row >> 1) & 7)) << 4);
    }
    const elem_t *gp = gamma + 64 * (int64_t)k_begin + 8 * t_chunk, *bp = beta + 64 * (int64_t)k_begin + 8 * t_chunk;
    // checkpoint copy (workgroup 0 only): where the raw row goes, or null
    elem_t *ckpt[P];
#pragma unroll
    for (int q = 0; q < P; ++q) {
        ckpt[q] = nullptr;
        const int m = q * RPP + t_row;
        if (blockIdx.x == 0 && p.act_dst && m < B) {
            elem_t *dst = static_cast<elem_t *>(p.act_dst);
            if (p.pd.block_table) {
                int32_t entry;
                int r;
                paged_slot(p.pd, m, entry, r);
                if (r >= 0 && entry < 0 && ~entry < p.pd.P_act)
                    ckpt[q] = dst + ((((int64_t)~entry) << p.pd.blk_log2) + r) * d + 64 * (int64_t)k_begin + 8 * t_chunk;
            } else {
                ckpt[q] = dst + (int64_t)m * p.act_row_stride + 64 * (int64_t)k_begin + 8 * t_chunk;
            }
        }
    }

    float16_t acc[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[rb][r] = 0.f;
    float m1[P], m2[P], shift[P];
#pragma unroll
    for (int q = 0; q < P; ++q) { m1[q] = 0.f; m2[q] = 0.f; shift[q] = 0.f; }
    float Gp[4] = {0.f, 0.f, 0.f, 0.f}, Tp[4] = {0.f, 0.f, 0.f, 0.f};        // this lane's part of G, T of weight rows 8 j + g_row

#pragma unroll
    for (int q = 0; q < P; ++q) rp[q] += 64 * (int64_t)k_begin;             // this group's part of the row

    vec8_t sv[kDepth][4], av[kDepth][P], gv[kDepth], bv[kDepth];
    const int last = my_steps > 0 ? my_steps - 1 : 0;
    auto fetch = [&](int slot, int sc) {                   // tile pieces (L2) before the streamed rows (HBM): loads retire in order
        if (sc > last) sc = last;
        if (my_steps <= 0) sc = -k_begin + k_steps - 1;    // a group without steps re-reads the last step of the axis and uses nothing
        gv[slot] = *reinterpret_cast<const vec8_t *>(gp + 64 * sc);
        bv[slot] = *reinterpret_cast<const vec8_t *>(bp + 64 * sc);
#pragma unroll
        for (int q = 0; q < P; ++q) av[slot][q] = *reinterpret_cast<const vec8_t *>(rp[q] + 64 * sc);
#pragma unroll
        for (int j = 0; j < 4; ++j) sv[slot][j] = __builtin_nontemporal_load(reinterpret_cast<const vec8_t *>(sp[j] + 64 * sc));
    };
    // builds the tile of step sc (used only when sc < my_steps) from register slot `slot` into buffer `buf`.
    // (x - shift) and its product with gamma are formed in the storage type, two elements per instruction for fp16
    // (the shift is near the row's mean, so the difference is small and its rounding is that of the operand itself);
    // the moments are summed in fp32 from the rounded differences, so that they describe exactly the rows that enter
    // the product.
    const vec2_t ones = {(elem_t)1.f, (elem_t)1.f};
    auto put = [&](int slot, int buf, int sc) {
        const bool valid = sc < my_steps;
#pragma unroll
        for (int q = 0; q < P; ++q) {
            vec8_t o;
            if (is_row[q]) {
                const vec2_t sh = {(elem_t)shift[q], (elem_t)shift[q]};
                float t1 = m1[q], t2 = m2[q];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const vec2_t df = vec2_t{av[slot][q][2 * e], av[slot][q][2 * e + 1]} - sh;
                    t1 = Elem<DT>::dot2(df, ones, t1);
                    t2 = Elem<DT>::dot2(df, df, t2);
                    const vec2_t pr = df * vec2_t{gv[slot][2 * e], gv[slot][2 * e + 1]};
                    o[2 * e] = pr[0];
                    o[2 * e + 1] = pr[1];
                }
                if (valid) { m1[q] = t1; m2[q] = t2; }
                if (valid && ckpt[q]) *reinterpret_cast<vec8_t *>(ckpt[q] + 64 * sc) = av[slot][q];
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] = (elem_t)0.f;
            }
            *reinterpret_cast<vec8_t *>(tile + buf * RB * KB + t_wr[q]) = o;
        }
    };

#pragma unroll
    for (int u = 0; u < kDepth - 1; ++u) fetch(u, u);
    // the shift of every input row: the mean of its first 64 elements (the 8 lanes of a row hold them), the same in
    // every group; rounded to the storage type, in which it is subtracted.  Asked for behind the first steps' loads,
    // so that the call's start pays one memory latency, not two.
#pragma unroll
    for (int q = 0; q < P; ++q) {
        const vec8_t h = *reinterpret_cast<const vec8_t *>(rp[q] - 64 * (int64_t)k_begin);
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) s += (float)h[e];
#pragma unroll
        for (int off = 1; off < 8; off <<= 1) s += __shfl_xor(s, off, 64);
        shift[q] = is_row[q] ? (float)(elem_t)(s * (1.0f / 64.0f)) : 0.f;
    }
    put(0, 0, 0);
    __syncthreads();
    for (int s = 0; s < steps_g; s += kDepth) {            // steps_g is the same for every group: the barriers match
#pragma unroll
        for (int u = 0; u < kDepth; ++u) {
            const int sc = s + u;
            fetch((u + kDepth - 1) % kDepth, sc + kDepth - 1);
            if (sc < steps_g) {                            // uniform over the workgroup
                put((u + 1) % kDepth, (sc + 1) & 1, sc + 1);           // the tile of step sc + 1, for the next pass
                if (sc < my_steps) {                       // uniform over the group
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        *reinterpret_cast<vec8_t *>(my + wr_off[j]) = sv[u][j];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const vec2_t w2 = {sv[u][j][2 * e], sv[u][j][2 * e + 1]};
                            Gp[j] = Elem<DT>::dot2(w2, vec2_t{gv[u][2 * e], gv[u][2 * e + 1]}, Gp[j]);
                            Tp[j] = Elem<DT>::dot2(w2, vec2_t{bv[u][2 * e], bv[u][2 * e + 1]}, Tp[j]);
                        }
                    }
                    // operand fragments of k piece jj + 1 are read while the MFMAs of piece jj run (left to the
                    // compiler, every MFMA waits for its own LDS read)
                    vec8_t wf[2], af[2][RB];
                    auto read_piece = [&](int jj) {
                        wf[jj & 1] = *reinterpret_cast<const vec8_t *>(my + rd_off[jj]);
#pragma unroll
                        for (int rb = 0; rb < RB; ++rb)
                            af[jj & 1][rb] = *reinterpret_cast<const vec8_t *>(tile + ((sc & 1) * RB + rb) * KB + rd_off[jj]);
                    };
                    read_piece(0);
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj) {
                        if (jj + 1 < 4) read_piece(jj + 1);
                        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                        for (int rb = 0; rb < RB; ++rb) acc[rb] = Elem<DT>::mfma_32x32x16(af[jj & 1][rb], wf[jj & 1], acc[rb]);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
                __syncthreads();                           // tile sc + 1 is complete; tile sc is free for sc + 2
            }
        }
    }

    // ---- the groups' parts meet in LDS (the loop's blocks and tiles are dead: the last barrier has been passed).
    // Moments of the group's part of every input row (the 8 lanes of a row hold its 8 chunk columns) ...
#pragma unroll
    for (int q = 0; q < P; ++q) {
        float a = m1[q], b2 = m2[q];
#pragma unroll
        for (int off = 1; off < 8; off <<= 1) {
            a += __shfl_xor(a, off, 64);
            b2 += __shfl_xor(b2, off, 64);
        }
        const int m = q * RPP + t_row;
        if (t_chunk == 0) mom[grp * RB * 32 + m] = make_float2(a, b2);
    }
    // ... its part of G and T of the wavefront's 32 weight rows ...
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        float gsum = Gp[j], tsum = Tp[j];
#pragma unroll
        for (int off = 1; off < 8; off <<= 1) {
            gsum += __shfl_xor(gsum, off, 64);
            tsum += __shfl_xor(tsum, off, 64);
        }
        if (g_chunk == 0) {
            gt[(grp * 2 + 0) * NF + 32 * wg + 8 * j + g_row] = gsum;
            gt[(grp * 2 + 1) * NF + 32 * wg + 8 * j + g_row] = tsum;
        }
    }
    // ... and its accumulators (the first group keeps its own in registers)
    if (KS > 1 && grp > 0) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int r = 0; r < 16; ++r) red[((grp * NW + wg) * RB * 16 + rb * 16 + r) * 64 + lane] = acc[rb][r];
    }
    __syncthreads();
    // row statistics (threads of all groups share the rows)
    const float inv_d = 1.0f / (float)d;
    for (int m = tid; m < B; m += GT * KS) {
        float a = 0.f, b2 = 0.f;
        for (int g2 = 0; g2 < KS; ++g2) { a += mom[g2 * RB * 32 + m].x; b2 += mom[g2 * RB * 32 + m].y; }
        const float dm = a * inv_d;                                         // mean - shift
        const float var = fmaxf(__builtin_fmaf(-dm, dm, b2 * inv_d), 0.f);
        const float rstd = 1.0f / __builtin_sqrtf(var + p.eps);
        stats[m] = make_float2(rstd, -dm * rstd);
    }
    // where the K / V row of every input row starts (element offset of head 0, element 0), or -1: not stored
    const int head_stride = p.pd.block_table ? (p.head_dim << p.pd.blk_log2) : p.L_cap * p.head_dim;
    if (!is_q) {
        for (int m = tid; m < B; m += GT * KS) {
            int64_t base = -1;
            if (p.pd.block_table) {
                int32_t entry;
                int r;
                paged_slot(p.pd, m, entry, r);
                if (r >= 0 && entry >= 0 && entry < p.pd.P_kv) base = ((((int64_t)entry * p.n_heads) << p.pd.blk_log2) + r) * p.head_dim;
            } else {
                base = ((int64_t)m * p.n_heads * p.L_cap + p.tok_pos) * p.head_dim;
            }
            rowdst[m] = base;
        }
    }
    __syncthreads();
    if (grp > 0) return;                                   // the first group finishes; no barrier below
#pragma unroll
    for (int g2 = 1; g2 < KS; ++g2)
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[rb][r] += red[((g2 * NW + wg) * RB * 16 + rb * 16 + r) * 64 + lane];
    const int col = 32 * wg + ln;
    if (col >= n_rows) return;
    const int n = n0 + col;                                // feature inside its weight array
    float G = 0.f, Tb = (float)(is_q ? static_cast<const elem_t *>(p.bq)[n] : static_cast<const elem_t *>(p.bkv)[n]);
    for (int g2 = 0; g2 < KS; ++g2) { G += gt[(g2 * 2 + 0) * NF + col]; Tb += gt[(g2 * 2 + 1) * NF + col]; }
    elem_t *dst;
    int64_t row_stride = 0;
    if (is_q) {
        dst = static_cast<elem_t *>(p.q_out) + n;
        row_stride = d;
    } else {
        const int f = n < d ? n : n - d;
        const int h = f / p.head_dim, e = f % p.head_dim;
        dst = static_cast<elem_t *>(n < d ? p.K_dst : p.V_dst) + (int64_t)h * head_stride + e;
    }
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int m = 32 * rb + 8 * (r >> 2) + 4 * lh + (r & 3);
            if (m < B) {
                const float2 st = stats[m];
                const elem_t o = (elem_t)__builtin_fmaf(acc[rb][r], st.x, __builtin_fmaf(st.y, G, Tb));
                if (is_q) {
                    dst[(int64_t)m * row_stride] = o;
                } else {
                    const int64_t base = rowdst[m];
                    if (base >= 0) dst[base] = o;
                }
            }
        }
}

PagedDst paged_dst(const QkvArgs &a)
{
    return PagedDst{a.block_table, a.seq_len, a.store_mask, a.max_blocks, a.blk_log2, a.P_kv, a.P_act};
}

template <int RB, int NW, int KS, int kDepth, int DT>
hipError_t launch_fused(const QkvArgs &a, hipStream_t s)
{
    FusedArgs f;
    f.x = a.x; f.gamma = a.ln_w; f.beta = a.ln_b; f.Wq = a.Wq; f.Wkv = a.Wkv; f.bq = a.bq; f.bkv = a.bkv;
    f.q_out = a.q_out; f.K_dst = a.K_dst; f.V_dst = a.V_dst; f.act_dst = a.act_dst; f.act_row_stride = a.act_row_stride;
    f.B = a.B; f.d = a.d; f.n_heads = a.n_heads; f.head_dim = a.head_dim; f.L_cap = a.L_cap; f.tok_pos = a.tok_pos;
    f.eps = a.eps; f.pd = paged_dst(a);
    constexpr int rows = 32 * NW;
    f.q_blocks = (a.d + rows - 1) / rows;
    const int kv_blocks = a.K_dst ? (2 * a.d + rows - 1) / rows : 0;
    auto kern = qkv_fused_kernel<RB, NW, KS, kDepth, DT>;
    constexpr int lds = fused_lds_bytes<RB, NW, KS>();
    static_assert(lds <= 160 * 1024, "the workgroup must fit the LDS of a compute unit");
    static LdsOnce lds_once;
    const hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kern), lds, lds_once);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)(f.q_blocks + kv_blocks)), dim3(64 * NW * KS), lds, s, f);
    return hipGetLastError();
}

// The shapes of the workgroup per tile height, from timing the four benchmark layers cold (B = 32, d = 4096: 41 us
// with three launches before, 30 now; B = 64, d = 5120: 50 -> 52; B = 128, d = 7168: 103 -> 130; B = 64, d = 9216:
// 114 -> 110): (wavefronts per group, groups, steps in registers).  More steps in flight did not help (the step
// time grew with them), more wavefronts did.
template <int RB, int DT>
hipError_t launch_rb(const QkvArgs &a, hipStream_t s)
{
    if constexpr (RB == 1) return launch_fused<1, 2, 4, 4, DT>(a, s);
    else if constexpr (RB == 2) return a.d < 8192 ? launch_fused<2, 2, 4, 3, DT>(a, s) : launch_fused<2, 4, 2, 3, DT>(a, s);
    else return launch_fused<RB, 4, 2, 3, DT>(a, s);
}

template <int DT>
hipError_t launch_dt(const QkvArgs &a, hipStream_t s)
{
    switch ((a.B + 31) / 32) {                             // blocks of 32 input rows
    case 1: return launch_rb<1, DT>(a, s);
    case 2: return launch_rb<2, DT>(a, s);
    case 3: return launch_rb<3, DT>(a, s);
    case 4: return launch_rb<4, DT>(a, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace

hipError_t launch_qkv_current(const QkvArgs &a, hipStream_t s)
{
    if (a.B <= 0) return hipSuccess;
    if (a.B > kQkvMaxRows || a.d % 64 != 0 || a.d < 64) return hipErrorInvalidValue;
    if (a.block_table && (!a.seq_len || a.max_blocks <= 0 || a.blk_log2 < 4 || a.blk_log2 > 10 || a.P_kv < 0 || a.P_act < 0))
        return hipErrorInvalidValue;
    return a.dtype == 1 ? launch_dt<1>(a, s) : launch_dt<0>(a, s);
}

}  // namespace hk
