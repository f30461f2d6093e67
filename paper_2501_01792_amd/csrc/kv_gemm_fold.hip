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
// Kernel shape (CDNA4).  One workgroup per compute unit, resident for the whole launch (grid =
// number of compute units); it walks its share of the 256 x 256 output tiles.  4 wavefronts,
// 128 x 128 accumulators each (AGPRs), as 8 x 8 blocks of v_mfma_f32_16x16x32_f16: on fp16 operands with
// full mantissas the launch runs against the power limit, and this shape does 15 % more flops inside it
// than 32x32x16 (half the accumulator register traffic per flop).  The reduction axis advances in k blocks of 64; a k block
// of one operand is a "unit" of 256 rows x 128 bytes = 32 KiB, and the 160 KiB of LDS are a ring of
// 5 units through which the units of all the workgroup's tiles stream in consumption order
// (weights of block g, activations of block g, weights of block g+1, ...): the loads run
// across tile boundaries, so only the first tile of a workgroup sees a cold pipeline.
//   * Loads are buffer_load ... lds, 16 bytes per lane; the 8 lanes of an LDS row fetch one whole
//     128-byte line of a global row (half-line requests halve the useful rate of the L2 channels).
//     The XOR swizzle of the 16-byte chunk index, (row / 2) % 8, is applied on the global side; it
//     makes the 16-row x 4-chunk fragment reads (ds_read_b128) conflict-free.
//   * While k block g is consumed (2 sub-steps of k = 32, 64 MFMAs each per wavefront) the weights
//     of block g+2 are issued during its first half (into the ring's spare slot) and the activations of
//     block g+2 behind the barrier early in its second half, into a slot that barrier has just freed.
//     One barrier per k block.  The weights, which the eight XCDs all read and which miss their L2 more
//     often, get the longer flight.  The byte offsets of a tile's 8 + 8 loads are computed once per tile;
//     a load in the main loop costs its issue slot and no vector arithmetic.
//   * Fragments (8 + 8 per sub-step) are double-buffered in registers; every MFMA slot carries at most
//     one LDS read and one direct load.
//   * End of a tile: a row table (destination offset + statistics per row) is built in the one
//     slot that is free at that moment; accumulators are read out of the AGPRs four rows at a
//     time, combined with the statistics, rounded to fp16 and stored head-split, 8 consecutive
//     features (16 bytes) per store.  The next tile's first MFMAs start from a zero C operand instead
//     of cleared accumulators.
#include "hk_internal.h"
#include "elem.h"
#include "kv_gemm_common.h"

#include <type_traits>

namespace hk {
namespace {

using namespace gemm;

constexpr int FBM = 256, FBN = 256, FBK = 64;
constexpr int FNT = 256;                                    // 4 wavefronts, 2 x 2
constexpr int FWM = 128, FWN = 128, FTM = 8, FTN = 8;          // 8 x 8 MFMA blocks of 16 x 16 per wavefront
constexpr int kSlots = 5;
constexpr int kRowBytes = FBK * 2;                          // 128-byte LDS rows: 8 chunks of 16 bytes
constexpr int kUnitBytes = 256 * kRowBytes;                 // 32 KiB: one operand of one k block
constexpr int kRingBytes = kSlots * kUnitBytes;             // 160 KiB
constexpr int kLoadsPerUnit = 8;                            // direct loads one lane issues per unit
// Order of the two units of a k block in the ring.  The first unit of block g + 2 is fetched early (during block g's
// first half, into the ring's one spare slot), the second late (behind block g's barrier, into a slot that barrier
// frees) and has the shorter time to land.
constexpr bool kWeightsFirst = true;

typedef __attribute__((address_space(3))) void *lds_ptr_t;

template <int DT>
struct Frags {
    typename Elem<DT>::V8 a[FTM], b[FTN];
};

__device__ __forceinline__ int next2(int s) { s += 2; return s >= kSlots ? s - kSlots : s; }

// Column block of the q-th MFMA of a sub-step (row block q / 8): odd row blocks run backwards, so that every MFMA
// shares one operand register set with the one before it, across row blocks too.  The sums are the same (every
// accumulator block still takes its k pieces in order); the launch runs against the power limit and the order with
// fewer operand changes is 0.5 % faster (63.38 -> 63.03 ms on the OPT-66B-shaped layer, three alternating runs).
__device__ __forceinline__ constexpr int snake(int q) { return ((q >> 3) & 1) ? 7 - (q & 7) : (q & 7); }


// acc[i][j][r] is MFMA block (i, j), register r: tile row wrow0 + 16 i + 4 (lane / 16) + r, output feature
// nb + j with nb = n0 + wcol0 + TN * (lane % 16): a lane holds TN = 8 consecutive features of every row.
template <int DT, int TM, int TN>
__device__ __forceinline__ void store_tile(const float4_t (&acc)[TM][TN], int lane, const RowDst *tab,
                                                  int wrow0, int nb, int d, int head_dim, int L_cap,
                                                  const float (&cn)[TN], const float (&bn)[TN],
                                                  typename Elem<DT>::T *__restrict__ K_out, typename Elem<DT>::T *__restrict__ V_out)
{
    typedef typename Elem<DT>::T elem_t;
    typedef typename Elem<DT>::V8 half8_t;
    static_assert(TN == 8, "one 16-byte store per row");
    if (nb >= 2 * d) return;
    const bool is_v = nb >= d;
    const int nn = is_v ? nb - d : nb;
    const int h = nn / head_dim, e = nn % head_dim;
    elem_t *dst_base = (is_v ? V_out : K_out) + ((int64_t)h * L_cap * head_dim + e);
    const RowDst *my = tab + wrow0 + 4 * (lane >> 4);
    // groups of 4 consecutive rows (one block row); the table rows of the next group are fetched while the
    // current group is converted and stored
    RowDst rows[2][4];
#pragma unroll
    for (int k = 0; k < 4; ++k) rows[0][k] = my[k];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        if (i + 1 < TM) {
#pragma unroll
            for (int k = 0; k < 4; ++k) rows[(i + 1) & 1][k] = my[(i + 1) * 16 + k];
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const RowDst row = rows[i & 1][r];
            half8_t v;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                float a;                                   // read in place, in this order: left to itself the compiler
                asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(a) : "a"(acc[i][j][r]));   // reads ahead and spills
                v[j] = (elem_t)__builtin_fmaf(a, row.rstd, __builtin_fmaf(row.nmr, cn[j], bn[j]));
            }
            __builtin_nontemporal_store(v, reinterpret_cast<half8_t *>(dst_base + row.base));
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

template <int GROUP_M, int DT>
__global__ __launch_bounds__(FNT) void kv_gemm_fold_kernel(
    const typename Elem<DT>::T *__restrict__ act, const float2 *__restrict__ stats,
    const typename Elem<DT>::T *__restrict__ Wp, const float *__restrict__ cvec, const float *__restrict__ bvec,
    typename Elem<DT>::T *__restrict__ K_out, typename Elem<DT>::T *__restrict__ V_out,
    int64_t M, int d, int n_heads, int head_dim, int L_act, int L_cap, int tok_off,
    int tiles_m, int tiles_n)
{
    extern __shared__ __align__(16) unsigned char smem[];
    typedef typename Elem<DT>::T elem_t;
    typedef typename Elem<DT>::V8 half8_t;

    const int N = 2 * d;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;

    const int n_tiles = tiles_m * tiles_n;
    const int my_tiles = (n_tiles - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x;   // >= 1: grid <= n_tiles
    const int nks = d / FBK;                                   // host guarantees d % 64 == 0 and nks >= 2

    // ---- direct-load roles.  One load of a wavefront fills 8 consecutive 128-byte LDS rows (1 KiB): lane l
    // writes row l / 8, physical chunk l % 8, and fetches the logical chunk (l % 8) ^ ((row / 2) % 8) of that
    // row, so that the 8 lanes of a row fetch one whole 128-byte line.  Load i of wavefront w covers LDS
    // rows 8 (w + 4 i) .. + 7; (row / 2) % 8 = (4 (w % 2) + l / 16) % 8 for all of them.
    const int l_row = lane >> 3;
    const int l_chunk = (lane & 7) ^ ((4 * (wave & 1) + (lane >> 4)) & 7);
    const int a_voff0 = ((8 * wave + l_row) * d + l_chunk * 8) * 2;          // activation row 8 w + l/8 (+ 32 i)
    // LDS row rho = 8 (w + 4 i) + l/8 of the weight unit belongs to wavefront column rho / 128, MFMA block
    // j = (rho % 128) / 16, block column c = rho % 16, and holds weight row 128 (rho / 128) + 8 c + j (so that a lane
    // ends up with 8 consecutive features): 64 (w % 2) + w / 2 + 8 (l/8)  (+ 128 (i/4) + 2 (i%4))
    const int b_voff0 = ((64 * (wave & 1) + (wave >> 1) + 8 * l_row) * d + l_chunk * 8) * 2;
    const int dma_wave = wave * 1024;                                        // + 4096 i, + slot

    // state of the load cursor: the k block whose units are issued next
    __amdgpu_buffer_rsrc_t a_rsrc, b_rsrc;
    // Byte offsets of this lane's 8 + 8 loads of a unit inside the tile's row panels, rows past the end clamped to
    // the last valid row: worked out once per tile, so that a load in the main loop costs no vector arithmetic (the
    // position along the reduction axis travels in the scalar offset).
    int a_voff[kLoadsPerUnit], b_voff[kLoadsPerUnit];
    int ld_kb = 0, ld_step = 1;
    auto set_load_tile = [&](int j) {
        int tm, tn;
        tile_coords<GROUP_M>((int)blockIdx.x + j * (int)gridDim.x, tiles_m, tiles_n, tm, tn);
        const int64_t m0 = (int64_t)tm * FBM;
        const int n0 = tn * FBN;
        int64_t a_bytes = (M - m0) * (int64_t)d * 2, b_bytes = ((int64_t)N - n0) * d * 2;
        if (a_bytes > 0x7fffffff) a_bytes = 0x7fffffff;        // a tile spans < 2^30 bytes
        if (b_bytes > 0x7fffffff) b_bytes = 0x7fffffff;
        a_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<elem_t *>(act + m0 * (int64_t)d), 0, (int)a_bytes, 0x00020000);
        b_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<elem_t *>(Wp + (int64_t)n0 * d), 0, (int)b_bytes, 0x00020000);
        const int ra = (M - m0 < FBM) ? (int)(M - m0) - 1 : FBM - 1;
        const int rb = (N - n0 < FBN) ? (N - n0) - 1 : FBN - 1;
        const int a_vmax = (ra * d + l_chunk * 8) * 2, b_vmax = (rb * d + l_chunk * 8) * 2;
#pragma unroll
        for (int i = 0; i < kLoadsPerUnit; ++i) {
            const int va = a_voff0 + i * 32 * d * 2;
            const int vb = b_voff0 + ((i >> 2) * 128 + 2 * (i & 3)) * d * 2;
            a_voff[i] = va < a_vmax ? va : a_vmax;
            b_voff[i] = vb < b_vmax ? vb : b_vmax;
        }
    };
    // The cursor runs two k blocks ahead of the MFMAs, so it leaves a tile before that tile's last two k blocks are
    // consumed: the switch is made there, once per tile, and the main loop over k blocks carries no branch for it
    // (a taken branch costs a single resident wavefront an instruction-fetch bubble).  After the workgroup's last
    // tile the cursor stays on that tile's last k block: the loads go on, unconditionally, into slots nobody reads.
    auto next_load_tile = [&](int c_j) {
        const bool more = c_j + 1 < my_tiles;                 // uniform
        if (more) set_load_tile(c_j + 1);
        ld_kb = more ? 0 : nks - 1;
        ld_step = more ? 1 : 0;
    };
    auto issue_a = [&](int slot, int i) {
        unsigned char *dst = smem + slot * kUnitBytes + dma_wave + i * 4096;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(a_rsrc, (lds_ptr_t)dst, 16, a_voff[i], ld_kb * (FBK * 2), 0, 0);
    };
    auto issue_b = [&](int slot, int i) {
        unsigned char *dst = smem + slot * kUnitBytes + dma_wave + i * 4096;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(b_rsrc, (lds_ptr_t)dst, 16, b_voff[i], ld_kb * (FBK * 2), 0, 0);
    };

    // ---- fragment reads: row (lane % 16) + 16 i of the wavefront's sub-tile, logical chunk 4 ks + lane / 16
    const int fr = lane & 15, fc = lane >> 4;
    int frag_off[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) frag_off[ks] = fr * kRowBytes + (((4 * ks + fc) ^ ((fr >> 1) & 7)) << 4);
    const int a_rd_wave = wm * FWM * kRowBytes;
    const int b_rd_wave = wn * FWN * kRowBytes;
    // The reads of a sub-step in the order its MFMAs need them: a[0], b[0..7], a[1..7].
    // which = 0: a[0]; 1..8: b[which - 1]; 9..15: a[which - 8]
    auto read_frag = [&](Frags<DT> &f, int sa, int sb, int ks, int which) {
        if (which == 0 || which > 8) {
            const int i = which == 0 ? 0 : which - 8;
            f.a[i] = *reinterpret_cast<const half8_t *>(smem + sa * kUnitBytes + a_rd_wave + frag_off[ks] + i * (16 * kRowBytes));
        } else {
            const int j = which - 1;
            f.b[j] = *reinterpret_cast<const half8_t *>(smem + sb * kUnitBytes + b_rd_wave + frag_off[ks] + j * (16 * kRowBytes));
        }
    };

    Frags<DT> f0, f1;

    // ---- prologue: k blocks 0 and 1 in flight (units 0..3 -> slots 0..3), block 0 landed, its first fragments read
    set_load_tile(0);
#pragma unroll
    for (int s = 0; s < 2; ++s) {
#pragma unroll
        for (int i = 0; i < kLoadsPerUnit; ++i) kWeightsFirst ? issue_b(2 * s, i) : issue_a(2 * s, i);
#pragma unroll
        for (int i = 0; i < kLoadsPerUnit; ++i) kWeightsFirst ? issue_a(2 * s + 1, i) : issue_b(2 * s + 1, i);
        ++ld_kb;
    }
    asm volatile("s_waitcnt vmcnt(16)" ::: "memory");
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int q = 0; q < 16; ++q) read_frag(f0, kWeightsFirst ? 1 : 0, kWeightsFirst ? 0 : 1, 0, q);

    int s1 = 0, s2 = 1;                                        // slots of the first and the second unit of k block g
    for (int c_j = 0; c_j < my_tiles; ++c_j) {                 // tiles of this workgroup
    float4_t acc[FTM][FTN];
    // one k block; `first`: the tile's first block, whose first MFMAs start from zero accumulators
    auto stage = [&](auto first) {
        constexpr bool FIRST = decltype(first)::value;
        const float4_t zero = {0.f, 0.f, 0.f, 0.f};
        const int n1 = next2(s1), n2 = next2(s2);              // k block g + 1
        const int early = next2(n1), late = s1;                // k block g + 2: units 2g+4 (the spare slot), 2g+5 (block g's first)
        const int sA = kWeightsFirst ? s2 : s1, sB = kWeightsFirst ? s1 : s2;
        const int sA1 = kWeightsFirst ? n2 : n1, sB1 = kWeightsFirst ? n1 : n2;
        // ---- sub-step 0 (f0, k 0..31): fragments of sub-step 1 -> f1; first unit of block g+2
#pragma unroll
        for (int q = 0; q < 64; ++q) {
            if (q == 0) __builtin_amdgcn_s_waitcnt(0xC07F);    // lgkmcnt(0): every fragment of f0, read long ago, in one wait
            const int qi = q >> 3, qj = snake(q);
            acc[qi][qj] = Elem<DT>::mfma_16x16x32(f0.a[qi], f0.b[qj], FIRST ? zero : acc[qi][qj]);
            if (q < 32 && (q & 1) == 0) read_frag(f1, sA, sB, 1, q >> 1);
            if ((q & 7) == 7) kWeightsFirst ? issue_b(early, q >> 3) : issue_a(early, q >> 3);
            __builtin_amdgcn_sched_barrier(0);
        }
        // ---- sub-step 1 (f1, k 32..63): wait + barrier; fragments of sub-step 0 of block g+1 -> f0; second unit of block g+2
#pragma unroll
        for (int q = 0; q < 64; ++q) {
            if (q == 0) __builtin_amdgcn_s_waitcnt(0xC07F);    // lgkmcnt(0): likewise f1
            const int qi = q >> 3, qj = snake(q);
            acc[qi][qj] = Elem<DT>::mfma_16x16x32(f1.a[qi], f1.b[qj], acc[qi][qj]);
            if (q == 3) {
                // Every LDS read of block g has come back (the wait at the top of this sub-step).  Wait for this
                // wavefront's loads of block g+1 (the 8 early loads of block g+2 may fly), then meet the others: after
                // the barrier block g+1 is complete in LDS and the slots of block g may be refilled.
                asm volatile("s_waitcnt vmcnt(8)\n\ts_barrier" ::: "memory");
            }
            if (q >= 4 && q < 36 && (q & 1) == 0) read_frag(f0, sA1, sB1, 0, (q - 4) >> 1);
            if (q >= 7 && (q & 7) == 7) kWeightsFirst ? issue_a(late, q >> 3) : issue_b(late, q >> 3);   // q = 7, 15, .., 63: loads 0..7
            __builtin_amdgcn_sched_barrier(0);
        }
        ld_kb += ld_step;
        s1 = n1; s2 = n2;
    };
    if (nks == 2) next_load_tile(c_j);                         // a tile of two k blocks: its first is its last but one
    stage(std::true_type{});                                   // k block 0 (loads: k block 2)
    {                                                          // k blocks 1 .. nks - 3 (loads: k blocks 3 .. nks - 1 of this tile),
        int c_kb = 1;                                          // two per pass: one taken branch per two k blocks
        for (; c_kb + 1 < nks - 2; c_kb += 2) {
            stage(std::false_type{});
            stage(std::false_type{});
        }
        if (c_kb < nks - 2) stage(std::false_type{});
    }
    if (nks > 2) {
        next_load_tile(c_j);
        stage(std::false_type{});                              // k block nks - 2 (loads: k block 0 of the next tile)
    }
            // ---- end of a tile: LayerNorm statistics, constants of the layer, fp16, head split.
            // What the epilogue needs from memory (the row's statistics, the constants of this lane's output
            // features) is asked for before the tile's last k block, whose MFMAs hide the latency; these
            // loads are older than the last block's early loads, so its vmcnt(8) covers them.
            static_assert(FBM == FNT, "one table row per thread");
            int tm, tn;
            tile_coords<GROUP_M>((int)blockIdx.x + c_j * (int)gridDim.x, tiles_m, tiles_n, tm, tn);
            const int64_t m0 = (int64_t)tm * FBM;
            const int n0 = tn * FBN;
            // Tile rows past the last token stand for the last token: their operand loads were clamped to its row, so
            // their accumulators equal its accumulators bit for bit, and they store the same bytes to the same place.
            // The write-out then needs no test per row (a branch per row costs more than the row's arithmetic).
            const int64_t m_row = m0 + tid < M ? m0 + tid : M - 1;
            const RowDst my_row = row_dst(m_row, M, n_heads, head_dim, L_act, L_cap, tok_off, stats);
            const int nb = n0 + wn * FWN + FTN * (lane & 15);
            float cn[FTN], bn[FTN];
#pragma unroll
            for (int j = 0; j < FTN; ++j) {
                cn[j] = nb < N ? cvec[nb + j] : 0.f;
                bn[j] = nb < N ? bvec[nb + j] : 0.f;
            }
    stage(std::false_type{});                                  // the last k block (loads: k block 1 of the next tile)
        {
            // The slot that held the second unit of the block just consumed is free until the next
            // block's late loads are issued: it holds the row table meanwhile.
            const int s_tab = s2 >= 2 ? s2 - 2 : s2 + kSlots - 2;        // slot of the second unit of block g
            RowDst *tab = reinterpret_cast<RowDst *>(smem + s_tab * kUnitBytes);
            tab[tid] = my_row;
            // Barriers that wait for LDS traffic only: __syncthreads() would also wait for every global access in
            // flight, i.e. for the next tile's first k blocks (two memory latencies per tile) and for the stores.
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
            store_tile<DT, FTM, FTN>(acc, lane, tab, wm * FWM, nb, d, head_dim, L_cap, cn, bn, K_out, V_out);
            asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");   // the table's slot is about to be refilled
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");           // loads issued past the end land before LDS is released
}

// One wavefront per output feature n: W'[n,:] = fp16(gamma * W[n,:]), c[n] = sum_k W'[n,k],
// b'[n] = b[n] + sum_k beta_k W[n,k]  (sums in fp32).
template <int DT>
__global__ __launch_bounds__(256) void prepare_layer_kernel(const typename Elem<DT>::T *__restrict__ W,
                                                            const typename Elem<DT>::T *__restrict__ bkv,
                                                            const typename Elem<DT>::T *__restrict__ ln_w,
                                                            const typename Elem<DT>::T *__restrict__ ln_b,
                                                            typename Elem<DT>::T *__restrict__ Wp, float *__restrict__ cvec,
                                                            float *__restrict__ bvec, int N, int d)
{
    const int lane = threadIdx.x & 63;
    const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (n >= N) return;                                        // whole wavefront leaves together; no barrier here
    typedef typename Elem<DT>::V8 half8_t;
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
            o[j] = (typename Elem<DT>::T)((float)w[j] * (float)gv[j]);
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

template <int DT>
hipError_t prepare_dt(const void *Wkv, const void *bkv, const void *ln_w, const void *ln_b,
                      void *Wp, float *cvec, float *bvec, int d, hipStream_t s)
{
    typedef typename Elem<DT>::T elem_t;
    const int N = 2 * d;
    hipLaunchKernelGGL(prepare_layer_kernel<DT>, dim3((unsigned)((N + 3) / 4)), dim3(256), 0, s,
                       static_cast<const elem_t *>(Wkv), static_cast<const elem_t *>(bkv),
                       static_cast<const elem_t *>(ln_w), static_cast<const elem_t *>(ln_b),
                       static_cast<elem_t *>(Wp), cvec, bvec, N, d);
    return hipGetLastError();
}

template <int DT>
hipError_t fold_dt(const KvGemmArgs &a, int grid, int tiles_m, int tiles_n, hipStream_t s)
{
    typedef typename Elem<DT>::T elem_t;
    auto kern = kv_gemm_fold_kernel<4, DT>;
    static_assert(kRingBytes == 160 * 1024, "the ring uses the whole 160 KiB LDS of a CU");
    static LdsOnce lds_once;
    hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kern), kRingBytes, lds_once);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(FNT), kRingBytes, s,
                       static_cast<const elem_t *>(a.act), a.stats,
                       static_cast<const elem_t *>(a.Wp), a.cvec, a.bvec,
                       static_cast<elem_t *>(a.K_out), static_cast<elem_t *>(a.V_out),
                       a.M, a.d, a.n_heads, a.head_dim, a.L_act, a.L_cap, a.tok_off, tiles_m, tiles_n);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_prepare_layer(const void *Wkv, const void *bkv, const void *ln_w, const void *ln_b,
                                void *Wp, float *cvec, float *bvec, int d, hipStream_t s, int dtype)
{
    return dtype == 1 ? prepare_dt<1>(Wkv, bkv, ln_w, ln_b, Wp, cvec, bvec, d, s)
                      : prepare_dt<0>(Wkv, bkv, ln_w, ln_b, Wp, cvec, bvec, d, s);
}

hipError_t launch_kv_gemm_fold(const KvGemmArgs &a, hipStream_t s)
{
    const int64_t tiles_m64 = (a.M + FBM - 1) / FBM;
    const int tiles_n = (2 * a.d + FBN - 1) / FBN;
    if (tiles_m64 * tiles_n > 0x7fffffffLL || a.d % FBK != 0 || a.d < 2 * FBK) return hipErrorInvalidValue;
    const int tiles_m = (int)tiles_m64;
    const int n_tiles = tiles_m * tiles_n;
    int dev = 0, cus = 0;
    const hipError_t e = current_device_cus(&dev, &cus);
    if (e != hipSuccess) return e;
    if (a.cu_limit > 0 && a.cu_limit < cus) cus = a.cu_limit;  // leave the rest of the chip to a kernel on another stream
    const int grid = n_tiles < cus ? n_tiles : cus;            // one resident workgroup per compute unit
    return a.dtype == 1 ? fold_dt<1>(a, grid, tiles_m, tiles_n, s) : fold_dt<0>(a, grid, tiles_m, tiles_n, s);
}

}  // namespace hk
