// Internal launch interface between the C-ABI layer (api.hip) and the gfx950 kernels.
// Everything here is host-callable; pointers are device pointers unless said otherwise.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

namespace hk {

// Host-side facts that do not change while the process lives, asked of the runtime once per device instead of
// on every launch (device_info.hip).
// The current device's ordinal and its number of compute units.
hipError_t current_device_cus(int *dev, int *cus);
// Raises the dynamic-LDS limit of `kernel` to `bytes` on the current device.  `once` belongs to the call site
// (one per kernel instantiation): the runtime call is made the first time the site runs on a device.
struct LdsOnce {
    std::atomic<uint64_t> done{0};     // bit i: set on device i
};
hipError_t allow_dynamic_lds(const void *kernel, int bytes, LdsOnce &once);

// Per-row LayerNorm statistics of act[M, d] (fp16, or bf16 with dtype 1) in fp32.
// stats[r] = (rstd_r, -mean_r * rstd_r), so that (x - mean) * rstd == fma(x, stats.x, stats.y).
hipError_t launch_ln_stats(const void *act, float2 *stats, int64_t M, int d, float eps, hipStream_t s, int dtype = 0);

struct KvGemmArgs {
    const void *act;       // [M, d] fp16
    const float2 *stats;   // [M]
    const void *ln_w;      // [d] fp16
    const void *ln_b;      // [d] fp16
    const void *Wkv;       // [2d, d] fp16
    const void *bkv;       // [2d] fp16
    const void *Wp;        // prepared layer (null when not given): [2d, d] fp16 gamma-scaled weights,
    const float *cvec;     //   [2d] row sums of Wp,
    const float *bvec;     //   [2d] bias with the LayerNorm bias folded in
    void *K_out;           // [B, H, L_cap, dh] fp16
    void *V_out;
    int64_t M;             // B * L_act
    int d, n_heads, head_dim;
    int L_act, L_cap, tok_off;
    int tile;              // 0 = choose, else 128 or 256
    int dtype;             // 0: fp16, 1: bf16 (bf16 always takes the 256 x 256 kernel)
    int cu_limit = 0;      // > 0: the persistent 256 x 256 kernel uses at most this many compute units (the others stay
                           // free for a kernel on another stream); 0: all of them
};
// LayerNorm-fused K/V projection: K_out/V_out rows <- LN(act) x Wkv^T + bkv, head-split.
hipError_t launch_kv_gemm(const KvGemmArgs &a, hipStream_t s);
// Whether launch_kv_gemm takes the 256 x 256 streaming kernel for this problem (tile: 0 = choose, 128, 256).
// That kernel works on a prepared layer (Wp, cvec, bvec), so the caller must supply one.
bool kv_gemm_uses_prepared(int64_t M, int d, int tile, int dtype = 0);
// The 256 x 256 kernel for prepared layers (LayerNorm folded around the product; needs Wp, cvec, bvec).
hipError_t launch_kv_gemm_fold(const KvGemmArgs &a, hipStream_t s);
// Fills Wp, cvec, bvec from the layer's parameters.
hipError_t launch_prepare_layer(const void *Wkv, const void *bkv, const void *ln_w, const void *ln_b,
                                void *Wp, float *cvec, float *bvec, int d, hipStream_t s, int dtype = 0);

struct AttnArgs {
    const void *q;         // [B, H, dh] fp16
    const void *K0, *V0;   // first token segment  [B*H, L0, dh] fp16 (may be null when L0 == 0)
    const void *K1, *V1;   // second token segment [B*H, L1, dh] fp16 (may be null when L1 == 0)
    int L0, L1;
    int BH;                // B * H
    int head_dim;          // 64 or 128
    float scale;           // multiplies q.k
    int n_waves;           // wavefronts that share the BH * (L0 + L1) token positions equally (attn_wavefronts)
    float *partial;        // [n_waves + BH, dh + 2] fp32
    void *out;             // [BH, dh] fp16
    float2 *lse;           // optional [BH]: (running maximum in the log2 domain, softmax denominator) of every pair
    hipEvent_t after_main; // optional: recorded after the streaming kernel, before the merge
    int dtype;             // 0: fp16, 1: bf16
};
// Wavefronts of the attention kernel that stay resident together on an MI355X: 256 compute units x
// 4 SIMDs x 4 wavefronts (the kernel's register footprint, <= 128 VGPRs, allows 4 per SIMD).
constexpr int kAttnResidentWaves = 256 * 4 * 4;
// The paged kernel carries block addressing on top and fits 3 wavefronts per SIMD.
constexpr int kPagedResidentWaves = 256 * 4 * 3;
constexpr int kAttnMaxWaves = 1 << 20;
// Number of wavefronts the attention kernel uses for BH pairs of L tokens; splits > 0 asks for
// that many token ranges per pair.  A function of the shape only, so that workspace sizes can be
// computed without a device.
int attn_wavefronts(int64_t BH, int64_t L, int splits, int resident = kAttnResidentWaves);
// Single-query attention over the two token segments taken as one context.
hipError_t launch_flash_decode(const AttnArgs &a, hipStream_t s);
// Joins the attention results of two disjoint token segments of the same (sequence, head) pairs: out_x [BH, dh]
// (16-bit) with lse_x [BH] = (maximum in the log2 domain, softmax denominator) each -> out [BH, dh].
hipError_t launch_segment_join(const void *out_a, const float2 *lse_a, const void *out_b, const float2 *lse_b, void *out,
                               int BH, int head_dim, int dtype, hipStream_t s);

struct QkvArgs {
    const void *x;         // [B, d] fp16: layer input of the current token of every sequence
    const void *ln_w, *ln_b;
    const void *Wq, *bq;   // [d, d], [d]
    const void *Wkv, *bkv; // [2d, d], [2d]
    void *q_out;           // [B, H, dh]
    void *K_dst, *V_dst;   // [B, H, L_cap, dh] or both null: no K/V row is produced
    void *act_dst;         // null, or where row b of x is copied: act_dst + b * act_row_stride (elements)
    int64_t act_row_stride;
    int B, d, n_heads, head_dim, L_cap, tok_pos;
    float eps;
    int dtype;             // 0: fp16, 1: bf16 (every 16-bit tensor above)
    // Write-back into a paged cache instead (block_table != nullptr): row b is token seq_len[b] - 1 of request b;
    // its logical block's table entry names the KV block (K_dst, V_dst are then the pools [P_kv, H, 2^blk_log2, dh])
    // or the ACT block (act_dst is then the pool [P_act, 2^blk_log2, d]) that takes the row.  Requests without
    // tokens and entries outside the pools are not written.
    const int32_t *block_table, *seq_len;
    const int32_t *store_mask;     // paged only, optional [B]: zero = the request's row is not stored (q is still produced)
    int max_blocks, blk_log2, P_kv, P_act;
};
constexpr int kQkvMaxRows = 128;       // rows one launch of the skinny kernel takes
// LayerNorm + Q (and K/V) projection of B <= kQkvMaxRows current-token rows, with write-back.
hipError_t launch_qkv_current(const QkvArgs &a, hipStream_t s);

struct PagedAttnArgs {
    const void *q;                     // [B, H, dh] fp16
    const void *K_pool, *V_pool;       // [P_kv, H, block_tokens, dh] fp16 (may be null when P_kv == 0)
    const void *K_regen, *V_regen;     // [P_act, H, block_tokens, dh] fp16: regenerated ACT blocks (null when P_act == 0)
    const int32_t *block_table;        // [B, max_blocks]: >= 0 KV block number, < 0 ACT block ~entry
    const int32_t *seq_len;            // [B] tokens per request
    const int64_t *cu_tokens;          // [B + 1] exclusive prefix sums of seq_len
    int64_t total_tokens;              // cu_tokens[B]
    int max_blocks, P_kv, P_act, block_tokens;
    int B, H, head_dim;
    float scale;
    int n_waves;                       // attn_wavefronts(H, total_tokens, 0) -- pairs' tokens counted as one line
    float *partial;                    // [n_waves + B H, dh + 2] fp32
    void *out;                         // [B, H, dh] fp16
    const int64_t *total_dev;          // optional (device): the sum of seq_len when only the device knows it; total_tokens
                                       // is then an upper bound (it sizes the launch)
    float2 *lse;                       // optional [B H]: (maximum in the log2 domain, denominator) of every pair; (., 0) when empty
    int dtype;                         // 0: fp16, 1: bf16 (q, the pools, out)
};
// Single-query attention of B requests of different lengths over a block-table-addressed hybrid cache.
hipError_t launch_paged_decode(const PagedAttnArgs &a, hipStream_t s);

struct AbsorbedArgs {
    const void *q;             // [B, H, dh]
    const void *act;           // [B, L_act, d]
    float4 *stats;             // [B * L_act] scratch: (rstd, mean, -(mean - first element) rstd, -) of every checkpoint row
    const void *Wp;            // prepared layer: [2d, d] gamma-scaled weights,
    const float *cvec, *bvec;  //   [2d] row sums of Wp, [2d] bias with the LayerNorm bias folded in
    void *U;                   // [H, B, d] fp16 scratch: the query carried through the key weights
    float *w_raw;              // [B, H, Lp] fp32 scratch: x_t . U  (Lp = absorbed_row_pitch(L_act))
    void *w;                   // [B, H, Lp] fp16 scratch: softmax weight times rstd, normalised; zero past L_act
    float4 *sums;              // [B, H] scratch: (maximum, sum p, sum w mean, -)
    void *Y;                   // [B, H, d] fp16 scratch: weighted sum of the raw checkpoint rows
    const void *out_c;         // [B, H, dh]: attention over the cached segment alone (unused when L_kv == 0)
    const float2 *lse_c;       // [B, H]: its (maximum, denominator)
    void *out;                 // [B, H, dh]
    float *proj_part;          // optional scratch [parts, min(B, kAbsorbMaxBatch), d] fp32 (absorbed_project_parts): with it large
    size_t proj_part_floats;   //   layers take the projection that cuts the reduction axis over workgroups; its capacity
    int B, H, head_dim, d, L_act, L_kv;
    int dt;                    // storage type of q, act, Wp, out_c, out (0: fp16, 1: bfloat16); the scratch vectors are fp16
    float scale, eps;
};
constexpr int kAbsorbMaxHeads = 128;   // heads (rows of the small operand of the score product) per sequence
constexpr int kAbsorbMaxBatch = 128;   // sequences one launch of the output projection takes
int absorbed_row_pitch(int L_act);     // elements between the rows of w_raw and w
void absorbed_project_parts(int d, int H, int *parts, int *steps_per_part);   // how the output projection cuts its reduction axis
// The checkpoint part of the decode attention without regenerating K/V (see absorbed.hip).
hipError_t launch_absorbed(const AbsorbedArgs &a, hipStream_t s);

struct PagedAbsorbedArgs {
    AbsorbedArgs abs;                  // act = the activation pool [P_act, block_tokens, d]; L_act = max_blocks * block_tokens
    const int32_t *block_table;        // [B, max_blocks]: < 0: checkpoint block ~entry
    const int32_t *seq_len;            // [B]
    int max_blocks, block_tokens, n_act_used;
    int32_t *list;                     // [B, max_blocks] scratch: the checkpoint blocks of every request in logical order
    int32_t *count, *last_rows, *n_rows;   // [B] scratch each: their number, the rows of the last one, the request's checkpoint rows
    int32_t *kv_table;                 // [B, max_blocks] scratch: the KV blocks of every request in logical order
    int32_t *kv_len;                   // [B] scratch: the request's cached tokens
    int64_t *kv_cu;                    // [B + 1] scratch: their prefix sums
};
// The same over a paged cache: launch_paged_index builds the two views of the block table (checkpoint blocks, KV
// blocks), the caller runs launch_paged_decode over the KV view (total_dev = kv_cu + B), launch_paged_absorbed does
// the checkpoint part and the join.
struct PagedAppendArgs {
    int32_t *block_table;              // [B, max_blocks]
    int32_t *seq_len;                  // [B]
    int64_t *cu_tokens;                // [B + 1]
    int32_t *counters;                 // [4]: KV blocks in use, ACT blocks in use, requests that could not grow (running sum), -
    const int32_t *active;             // optional [B]: nonzero = the request takes a token
    int32_t *grew;                     // optional [B], written: 1 = the request took its token, 0 = it did not (inactive or stuck)
    int B, max_blocks, block_tokens, P_kv, P_act;
    int64_t act_host, kv_host;         // the ratio every request keeps (Eq. 11)
};
// One token more for every active request, with the block bookkeeping that goes with it (see paged_append.hip).
hipError_t launch_paged_append(const PagedAppendArgs &a, hipStream_t s);
hipError_t launch_paged_index(const PagedAbsorbedArgs &a, hipStream_t s);
hipError_t launch_paged_absorbed(const PagedAbsorbedArgs &a, hipStream_t s);

}  // namespace hk
