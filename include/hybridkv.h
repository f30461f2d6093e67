/*
 * hybridkv -- C ABI of the per-layer hybrid-cache decode step on AMD MI355X (gfx950).
 *
 * The step is the "KV Gen -> concat -> MHA" slice of the execution engine of
 * arXiv 2501.01792 (Sec. 4.2.2): keys and values of the context tokens that
 * are held as activation checkpoints are regenerated from those checkpoints
 * (Sec. 3.3, Eq. 7), joined with the keys and values that are held directly
 * in the KV cache (Eq. 3), and the decode query of each sequence attends over
 * the union (Eq. 4).
 *
 * Conventions common to every call
 *   - Every data pointer is a DEVICE pointer owned by the caller and must be
 *     16-byte aligned.  hk_shape / hk_layer_params themselves are HOST structs
 *     passed by pointer and read before the call returns.
 *   - Storage dtype is IEEE fp16 (HK_DTYPE_F16), the precision of the paper's
 *     models (Sec. 5.1); accumulation is fp32.  Every device entry point and
 *     size query also takes bfloat16 (HK_DTYPE_BF16: every fp16 tensor below is
 *     bf16 instead).
 *   - The library allocates nothing.  Scratch memory is the caller's
 *     `workspace` (device, 256-byte aligned, at least hk_workspace_bytes()).
 *   - Calls enqueue work on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and return without synchronising.  Calls that share a
 *     workspace must be ordered by the caller (same stream, or events).
 *   - Return value: HK_OK (0) or a negative hk_status.  All argument checks run
 *     on the host before anything is launched, so a rejected call has touched
 *     no device memory.
 *
 * Tensor layouts (row-major, last index fastest)
 *   act      [B, L_act, d]     activation checkpoints A_c: the layer's input
 *                              hidden states of the tokens not held as KV
 *   ln_w, ln_b [d]             LayerNorm weight and bias of the layer's
 *                              pre-attention LayerNorm
 *   Wkv      [2d, d]           fused projection, "output feature x input":
 *                              rows 0..d-1 are the columns of W_K, rows d..2d-1
 *                              the columns of W_V in Eq. 7
 *   bkv      [2d]              K bias, then V bias
 *   K, V     [B, H, L, dh]     head-major: one (sequence, head) is one
 *                              contiguous L*dh run; feature n of a token is
 *                              head n / dh, element n % dh
 *   q, out   [B, H, dh]        (= [B, d])
 */
#ifndef HYBRIDKV_H
#define HYBRIDKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum hk_status {
    HK_OK = 0,
    HK_ERR_NULL = -1,      /* a required pointer is NULL */
    HK_ERR_SHAPE = -2,     /* d != n_heads*head_dim, head_dim not in {64,128}, negative or overflowing sizes */
    HK_ERR_RATIO = -3,     /* ratio outside [0,1] or inconsistent with L_kv, L_act */
    HK_ERR_ALIGN = -4,     /* a data pointer is not 16-byte aligned (workspace: 256) */
    HK_ERR_WORKSPACE = -5, /* workspace_bytes smaller than hk_workspace_bytes() */
    HK_ERR_DTYPE = -6,     /* a dtype the entry point does not take */
    HK_ERR_LAUNCH = -7,    /* the HIP runtime reported an error at launch */
    HK_ERR_STATIC_LIMIT = -8 /* hk_hybrid_decode_attn_static: the problem needs more than HK_STATIC_SCRATCH_BYTES of scratch */
} hk_status;

enum { HK_DTYPE_F16 = 0, HK_DTYPE_BF16 = 1 };

/* Shape and numerics of one decoder layer.  Host struct. */
typedef struct hk_shape {
    int32_t d;             /* hidden size */
    int32_t n_heads;       /* H */
    int32_t head_dim;      /* dh, 64 or 128; d == n_heads * head_dim */
    int32_t dtype;         /* HK_DTYPE_F16 or HK_DTYPE_BF16 */
    float ln_eps;          /* LayerNorm epsilon (inside the square root); OPT uses 1e-5 */
    float softmax_scale;   /* multiplies q.k before the softmax; <= 0 selects head_dim^-1/2 */
    int32_t attn_splits;   /* attention work split: 0 lets the library choose (the tokens of all
                              (sequence, head) pairs are shared equally among the wavefronts that are
                              resident at once); 1..HK_MAX_SPLITS asks for that many equal token ranges
                              per pair */
    int32_t gemm_tile;     /* output tile edge of the projection kernel: 0 lets the library
                              choose, otherwise 128 or 256 */
} hk_shape;

enum { HK_MAX_SPLITS = 64 };

/* Device pointers to the parameters the step needs from one decoder layer. */
typedef struct hk_layer_params {
    const void *ln_w;      /* [d]     */
    const void *ln_b;      /* [d]     */
    const void *Wkv;       /* [2d, d] */
    const void *bkv;       /* [2d]    */
    const void *prepared;  /* NULL, or the buffer hk_prepare_layer filled from these four */
} hk_layer_params;

/*
 * Bytes of device workspace that hk_hybrid_decode_attn needs for a batch of B
 * sequences with L_kv cached and L_act checkpointed tokens each (the
 * regenerated K/V, per-row LayerNorm statistics, room for a per-call prepared
 * layer when the regeneration is large, and the attention partials for
 * shape->attn_splits).  Returns 0 when the shape is invalid.
 */
size_t hk_workspace_bytes(const hk_shape *shape, int32_t B, int32_t L_kv, int32_t L_act);

/*
 * Bytes of device workspace that hk_regen_kv needs (per-row LayerNorm
 * statistics, and room for a per-call prepared layer when the regeneration is
 * large).  Returns 0 when the shape is invalid.
 */
size_t hk_regen_workspace_bytes(const hk_shape *shape, int32_t B, int32_t L_act);

/*
 * Optional one-time preparation of a layer (its parameters are fixed during
 * inference).  Eq. 7 applied to LayerNorm-ed checkpoints can be regrouped as
 *     [K V][t, n] = rstd_t * (a_t . W'[n, :]) - mean_t * rstd_t * c[n] + b'[n],
 *     W'[n, k] = ln_w[k] * Wkv[n, k],  c[n] = sum_k W'[n, k],  b'[n] = bkv[n] + sum_k ln_b[k] * Wkv[n, k],
 * which lets the raw checkpoint rows feed the matrix cores while the row
 * statistics are applied to the accumulators.  hk_prepare_layer computes W'
 * (fp16), c and b' (fp32) into `prepared` (device, 256-byte aligned, at least
 * hk_prepared_bytes(shape) bytes, owned by the caller, valid as long as it is
 * referenced from hk_layer_params.prepared).  Large regenerations run on this
 * form.  A call that is not given a prepared layer prepares one itself, in its
 * workspace, every time (one extra pass over the weights); a caller that keeps
 * the layer prepared saves that pass.  Small regenerations apply the LayerNorm
 * on the fly instead and ignore `prepared`.
 */
size_t hk_prepared_bytes(const hk_shape *shape);
int hk_prepare_layer(const hk_shape *shape, const hk_layer_params *params,
                     void *prepared, size_t prepared_bytes, void *stream);

/*
 * "KV Gen" (Sec. 4.2.2; Sec. 3.3, Eq. 7): regenerate keys and values from
 * activation checkpoints,
 *     [K V] = LayerNorm(act; ln_w, ln_b, ln_eps) x [W_K W_V] + [b_K b_V],
 * skipping everything the layer does after QKV generation.  The LayerNorm is
 * the layer's own pre-attention one: a checkpoint is the layer's input tensor.
 *
 *   act          [B, L_act, d] fp16, read only
 *   K_out, V_out [B, H, L_cap, dh] fp16; token t of sequence b is written to
 *                row tok_off + t of every head of b, other rows are untouched
 *                (0 <= tok_off, tok_off + L_act <= L_cap)
 *   workspace    needs hk_regen_workspace_bytes(shape, B, L_act)
 * B == 0 or L_act == 0 is a successful no-op.
 */
int hk_regen_kv(const hk_shape *shape,
                const void *act, int32_t B, int32_t L_act,
                const hk_layer_params *params,
                void *K_out, void *V_out, int32_t L_cap, int32_t tok_off,
                void *workspace, size_t workspace_bytes, void *stream);

/*
 * The whole step (Sec. 4.2.2; Eq. 7, 3, 4): regenerate K/V from `act`,
 * treat them as the continuation of the cached K/V along the token axis
 * (no copy is made), and compute for the one decode query of every
 * (sequence, head)
 *     out = softmax(softmax_scale * q K^T) V
 * over all L = L_kv + L_act context tokens.  No mask: the query attends to
 * every context token.  Softmax attention does not depend on token order, so
 * which tokens sit in which store does not matter.
 *
 *   q            [B, H, dh] fp16, unscaled
 *   K_cache, V_cache [B, H, L_kv, dh] fp16; may be NULL when L_kv == 0
 *   act          [B, L_act, d] fp16; may be NULL when L_act == 0
 *   ratio        fraction of the context held as KV; checked against the
 *                lengths: L_kv must equal round(ratio * (L_kv + L_act))
 *   out          [B, H, dh] fp16
 *   workspace    needs hk_workspace_bytes(shape, B, L_kv, L_act); on return
 *                (after the stream has run) its head holds the regenerated
 *                K [B,H,L_act,dh] then V [B,H,L_act,dh]
 * L_kv + L_act == 0 is rejected with HK_ERR_SHAPE (softmax over nothing).
 */
int hk_hybrid_decode_attn(const hk_shape *shape,
                          const void *q,
                          const void *K_cache, const void *V_cache, int32_t L_kv,
                          const void *act, int32_t L_act, int32_t B,
                          const hk_layer_params *params, float ratio,
                          void *out,
                          void *workspace, size_t workspace_bytes, void *stream);

/*
 * The step of hk_hybrid_decode_attn issued on two streams (Sec. 4.2.2: the engine overlaps KV generation with the
 * work that does not depend on it; inside one GPU that work is the attention over the cached segment).  On
 * `side_stream`: the attention of every query over the cached K/V alone.  On `stream`: the regeneration (Eq. 7), then
 * the attention over the regenerated rows alone.  The two results are joined on `stream` through their softmax
 * maxima and denominators (Eq. 3, 4 over the union).  Same result as hk_hybrid_decode_attn up to rounding (the two
 * segment outputs are rounded to the storage type before the join), not bit for bit; bit-identical to itself when
 * side_stream == stream.
 *   stream, side_stream   hipStream_t; side_stream may equal stream (then everything runs in order on it)
 *   fork_event, join_event  two hipEvent_t owned by the caller (the library creates nothing); the library records
 *                         fork on stream behind the LayerNorm statistics kernel (which is bound by HBM like the
 *                         attention: only the projection is worth running beside), makes side_stream wait for it,
 *                         records join on side_stream after its work
 *                         and makes stream wait for join: on return all later work on `stream` is ordered after
 *                         both parts, and side_stream is free again once join has completed
 *   gemm_cus              > 0: the persistent projection kernel occupies at most this many compute units, which
 *                         leaves the others to the side stream's kernel (it otherwise holds every compute unit's
 *                         registers and LDS, and the two kernels take turns); 0: all of them
 *   workspace             needs hk_two_stream_workspace_bytes(shape, B, L_kv, L_act)
 * With L_kv == 0 or L_act == 0 there is nothing to overlap and the call is hk_hybrid_decode_attn on `stream`.
 * Errors as for hk_hybrid_decode_attn; the events must not be NULL when both segments have tokens.
 */
size_t hk_two_stream_workspace_bytes(const hk_shape *shape, int32_t B, int32_t L_kv, int32_t L_act);
int hk_hybrid_decode_attn_two_stream(const hk_shape *shape,
                                     const void *q,
                                     const void *K_cache, const void *V_cache, int32_t L_kv,
                                     const void *act, int32_t L_act, int32_t B,
                                     const hk_layer_params *params, float ratio,
                                     void *out, void *workspace, size_t workspace_bytes,
                                     void *stream, void *side_stream, void *fork_event, void *join_event, int32_t gemm_cus);

/*
 * hk_hybrid_decode_attn for callers that cannot allocate and have no workspace to pass: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same step, same arguments minus the workspace,
 * same kernels, bit-identical result.  The scratch memory (regenerated K/V, row statistics, attention partials) is a
 * static device array inside the library, HK_STATIC_SCRATCH_BYTES per GPU, held by every GPU the library's code is
 * loaded on until the process ends.  The call allocates nothing and frees nothing.
 *   - A problem whose scratch need exceeds the array is refused with HK_ERR_STATIC_LIMIT before anything is launched.
 *     The need is hk_workspace_bytes(shape, B, L_kv, L_act), less hk_prepared_bytes(shape) when params->prepared is
 *     given (large regenerations run on a prepared layer; a caller that brings one saves the room for it -- with
 *     d = 4096 that room alone is 64 MiB, so large layers need a prepared layer here).
 *   - All calls on one GPU share that GPU's array: calls that overlap on one GPU (different streams, or threads)
 *     race on it; the caller orders them.  The array keeps the last call's contents; nothing in it needs clearing
 *     (every byte a kernel of the step reads has been written earlier in the same call).
 *   - The first call on a GPU looks the array's address up (no allocation; the runtime may load the library's code
 *     object then): make one call on a GPU before capturing the step into a graph there.
 */
enum { HK_STATIC_SCRATCH_BYTES = 32 << 20 };
int hk_hybrid_decode_attn_static(const hk_shape *shape,
                                 const void *q,
                                 const void *K_cache, const void *V_cache, int32_t L_kv,
                                 const void *act, int32_t L_act, int32_t B,
                                 const hk_layer_params *params, float ratio,
                                 void *out, void *stream);

/*
 * Where hk_hybrid_decode_attn leaves the regenerated rows: byte offsets, from the start of its workspace, of
 * K [B,H,L_act,dh] and of V [B,H,L_act,dh] (a test or a caller that wants to keep them reads them there after the
 * stream has run).  Host-only.  HK_OK or the status the step itself would give for the shape.
 */
int hk_regen_offsets(const hk_shape *shape, int32_t B, int32_t L_act, size_t *k_offset, size_t *v_offset);

/*
 * NOT A PRODUCT CALL: a measurement aid for benchmarks and profilers.
 * hk_hybrid_decode_attn with per-kernel time stamps: the same
 * step (Sec. 4.2.2; Eq. 7, 3, 4) and the same arguments, plus `events`, a HOST
 * array of n_events hipEvent_t handles (passed as void*; NULL entries are
 * skipped) owned by the caller.  The library records, on `stream`,
 *   events[0] before the first kernel,      events[1] after the LayerNorm statistics,
 *   events[2] after the K/V projection,     events[3] after the attention streaming kernel,
 *   events[4] after the merge of the attention partials (end of the step).
 * Stages that do not run (L_act == 0) leave their event recorded back to back
 * with the previous one.
 */
int hk_hybrid_decode_attn_marked(const hk_shape *shape,
                                 const void *q,
                                 const void *K_cache, const void *V_cache, int32_t L_kv,
                                 const void *act, int32_t L_act, int32_t B,
                                 const hk_layer_params *params, float ratio,
                                 void *out,
                                 void *workspace, size_t workspace_bytes, void *stream,
                                 void **events, int32_t n_events);

/*
 * QKV generation for the current input token of every sequence, and its write-back (Sec. 4.2.2: the
 * decode step generates Q, K, V of the input token, Eq. 2, and afterwards keeps the token either as
 * a KV entry or as an activation checkpoint):
 *     xhat = LayerNorm(x_cur; ln_w, ln_b, ln_eps)
 *     q    = xhat x W_Q + b_Q                       -> q_out
 *     k, v = xhat x [W_K W_V] + [b_K b_V]           -> row tok_pos of K_dst, V_dst   (when given)
 *     x_cur                                         -> row act_pos of act_dst        (when given)
 * A caller that keeps the token as a KV entry passes K_dst/V_dst = its cache and tok_pos = L_kv; one
 * that keeps it as a checkpoint passes act_dst = its checkpoint store and act_pos = L_act (the
 * token's K/V are then regenerated with the other checkpoints by hk_hybrid_decode_attn).  Either
 * way the token is in a store afterwards and the step attends over it like over any other.
 *
 *   x_cur     [B, d] fp16, read only
 *   params    ln_w, ln_b, Wkv [2d, d], bkv [2d] as everywhere (prepared is not used)
 *   Wq, bq    [d, d] (output feature x input) and [d], fp16
 *   q_out     [B, H, dh] fp16
 *   K_dst, V_dst [B, H, L_cap, dh] fp16, both NULL or both given; only row tok_pos is written
 *   act_dst   [B, act_cap, d] fp16 or NULL; only row act_pos is written
 *   workspace needs hk_qkv_workspace_bytes(shape, B) (a token amount: the call is a single kernel that keeps its
 *             intermediate values on chip; the argument is kept so that callers need not change)
 * B == 0 is a successful no-op.
 */
size_t hk_qkv_workspace_bytes(const hk_shape *shape, int32_t B);
int hk_qkv_current(const hk_shape *shape, const void *x_cur, int32_t B,
                   const hk_layer_params *params, const void *Wq, const void *bq,
                   void *q_out,
                   void *K_dst, void *V_dst, int32_t L_cap, int32_t tok_pos,
                   void *act_dst, int32_t act_cap, int32_t act_pos,
                   void *workspace, size_t workspace_bytes, void *stream);

/*
 * Paged hybrid cache (Sec. 4.1, 4.2.1): the context of every request is a list of logical blocks of
 * `block_tokens` tokens; a block is a KV block (K and V rows in the KV pool) or an ACT block (the
 * tokens' checkpoints in the activation pool, half the bytes).  The block table maps each logical block
 * to its kind and physical block number.  Everything lives in device memory (there is no host offload
 * on this path, so the table carries no location).
 *
 *   K_pool, V_pool [P_kv, H, block_tokens, dh] fp16     a KV block holds its tokens head-major
 *   act_pool       [P_act, block_tokens, d]    fp16     an ACT block holds its tokens' layer inputs
 *   block_table    [B, max_blocks] int32, device: entry >= 0 is KV block `entry`; entry < 0 is ACT
 *                  block ~entry (bitwise not).  Only the first ceil(seq_len[r] / block_tokens) entries of
 *                  row r are read.  ACT entries must be < n_act_used, KV entries < P_kv.
 *   seq_len        [B] int32, device: tokens of request r; the last block may be partly filled
 *   cu_tokens      [B + 1] int64, device: exclusive prefix sums of seq_len
 *   total_tokens   HOST copy of cu_tokens[B], or any upper bound of it: the library sizes its launch and its
 *                  workspace from it; the kernels read the lengths, the prefix sums and their total on the device
 *   n_act_used     ACT blocks 0 .. n_act_used - 1 of the pool are in use: they are the ones regenerated (an upper
 *                  bound regenerates blocks that no table names, which costs time and changes no result)
 */
typedef struct hk_paged_cache {
    const void *K_pool, *V_pool;
    const void *act_pool;
    const int32_t *block_table;
    const int32_t *seq_len;
    const int64_t *cu_tokens;
    int64_t total_tokens;
    int32_t P_kv, P_act, n_act_used;
    int32_t block_tokens;          /* a power of two, 16 .. 1024 */
    int32_t max_blocks;
} hk_paged_cache;

/*
 * hk_qkv_current with the write-back into a paged cache (Sec. 4.2.2 on the block layout of Sec. 4.1): the input
 * token of request r is token seq_len[r] - 1 of its context, i.e. seq_len already counts it and its logical
 * block has its entry in the table (which kind of block a new block is, is the caller's policy: Eq. 11,
 * hk_next_block_type).  Its K and V rows go to row (seq_len[r] - 1) % block_tokens of that KV block, or, when the
 * entry names an ACT block, its layer input x_cur[r] goes to that row of the ACT block.  q is produced for every
 * request.  The POOLS ARE WRITTEN by this call (one row of one block per request; the struct declares them const
 * for the calls that only read them); block_table and seq_len are read; cu_tokens, total_tokens and n_act_used
 * are not used.  A request with seq_len[r] == 0 and an entry outside its pool (KV: >= P_kv, ACT: >= P_act) are
 * not written.  store_mask ([B] int32, device, or NULL = store all): a request whose entry is zero gets its q
 * and NOTHING is written for it.  A decode loop passes the `grew` array of hk_paged_append here: a request that took
 * no token in this step (inactive, table row full, pool exhausted) still has seq_len[r] - 1 pointing at its last
 * CACHED token, which an unmasked call would overwrite with the current input.  K and V are not computed when there is no KV pool (P_kv == 0).  Other arguments, workspace
 * (hk_qkv_workspace_bytes) and errors as for hk_qkv_current; block_tokens not a power of two in 16 .. 1024 or
 * max_blocks <= 0: HK_ERR_SHAPE.  fp16 or bf16.
 */
int hk_qkv_current_paged(const hk_shape *shape, const void *x_cur, int32_t B,
                         const hk_layer_params *params, const void *Wq, const void *bq,
                         void *q_out, const hk_paged_cache *cache, const int32_t *store_mask,
                         void *workspace, size_t workspace_bytes, void *stream);

/*
 * The hybrid-cache decode step on a paged cache: regenerate the K/V rows of the ACT blocks in use
 * (Sec. 3.3, Eq. 7, over the whole activation pool prefix as one GEMM), then for the decode query of
 * every (request, head) attend over all of the request's tokens through the block table (Eq. 3, 4).
 * Requests may have different lengths; a request of length 0 gets an all-zero output.
 *
 *   q, out     [B, H, dh] fp16
 *   params     as for hk_hybrid_decode_attn (may be NULL when n_act_used == 0)
 *   workspace  needs hk_paged_workspace_bytes(shape, B, cache)
 * The table, lengths and prefix sums are device data and cannot be checked on the host; the kernels
 * clamp block numbers to the pools, so inconsistent tables give wrong numbers, not stray accesses.
 */
size_t hk_paged_workspace_bytes(const hk_shape *shape, int32_t B, const hk_paged_cache *cache);
int hk_paged_decode_attn(const hk_shape *shape, const void *q, int32_t B, const hk_paged_cache *cache,
                         const hk_layer_params *params, void *out,
                         void *workspace, size_t workspace_bytes, void *stream);

/*
 * The same step as hk_hybrid_decode_attn (Sec. 4.2.2; Eq. 7, 3, 4) with the same arguments and the same
 * result up to rounding, computed WITHOUT regenerating K/V: a comparison variant beyond the paper.
 * For one query per head the K projection of Eq. 7 is applied to the query instead of to the
 * checkpoint rows (score_t = x^_t . (W_K,h^T q_h) + q_h . b_K,h) and the V projection to the weighted
 * sum of the rows instead of to every row (o_h = W_V,h (sum_t p_t x^_t) + b_V,h), LayerNorm folded in as
 * in the prepared layer; the checkpoints are read twice, the weights once, and about head_dim times
 * fewer FLOP are spent.  The cached segment takes the ordinary attention kernel; the two segments are
 * joined through their softmax maxima and denominators.  Intermediate values that the regenerating path
 * rounds to fp16 (the K and V rows) are not rounded here and others are (the carried query, the
 * weighted row sum), so the two entry points agree to the tolerance of the step, not bit for bit.
 *
 *   n_heads <= 128, B <= 65535; otherwise HK_ERR_SHAPE.
 *   workspace    needs hk_absorbed_workspace_bytes(shape, B, L_kv, L_act); scratch only.
 * bfloat16 tensors are converted to fp16 as they are loaded and the step computes as it does for fp16 (the
 * carried query and the weighted row sum keep 11 significant bits); the conversion is exact for magnitudes
 * from 2^-14 to 65504, larger ones are taken as 65504.
 * A layer without `prepared` is prepared inside the call (one pass over the weights).
 */
size_t hk_absorbed_workspace_bytes(const hk_shape *shape, int32_t B, int32_t L_kv, int32_t L_act);
int hk_hybrid_decode_attn_absorbed(const hk_shape *shape,
                                   const void *q,
                                   const void *K_cache, const void *V_cache, int32_t L_kv,
                                   const void *act, int32_t L_act, int32_t B,
                                   const hk_layer_params *params, float ratio,
                                   void *out,
                                   void *workspace, size_t workspace_bytes, void *stream);

/*
 * hk_paged_decode_attn without regenerating K/V: the two ideas above together.  Same arguments and the same
 * result up to rounding as hk_paged_decode_attn (Sec. 4.1, 4.2.1; Eq. 7, 3, 4).  Every request's row of the
 * block table is split on the device into its KV blocks and its checkpoint blocks, each in logical order.  The
 * KV blocks take the block-table attention kernel; the checkpoint blocks take the steps of
 * hk_hybrid_decode_attn_absorbed (scores per block, softmax per request over its own number of checkpoint
 * rows, weighted row sum through the block list); the two parts are joined through their softmax maxima and
 * denominators.  A request without tokens gets an all-zero output.  n_heads <= 128, B <= 65535; workspace:
 * hk_paged_absorbed_workspace_bytes (scratch only; the table, seq_len and cu_tokens are not written).
 * When n_act_used > 0 every length and every table entry is read on the device at run time and cu_tokens is not
 * read at all; total_tokens (which sizes the launch and the workspace) may then be any upper bound of the sum of
 * seq_len, and n_act_used any upper bound up to P_act of the ACT blocks the table names.  With such bounds one
 * HIP graph that holds hk_qkv_current_paged and this call serves successive decode steps while only device
 * memory changes between its replays (new input rows, lengths, table entries).
 */
size_t hk_paged_absorbed_workspace_bytes(const hk_shape *shape, int32_t B, const hk_paged_cache *cache);
int hk_paged_decode_attn_absorbed(const hk_shape *shape, const void *q, int32_t B, const hk_paged_cache *cache,
                                  const hk_layer_params *params, void *out,
                                  void *workspace, size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------
 * Cache-management policy arithmetic (Sec. 4.3).  Host-only: every pointer below is a HOST pointer,
 * nothing touches a device.  Times are in any one unit, sizes in any one unit; block counts are real
 * numbers inside the models and whole blocks (rounded down) in the results.
 */

/* A linear time model T(n) = slope * n + offset over a block (or token) count n: the form the paper
 * fits to its samples of T_kv_gen and T_load_kv (Sec. 4.3, the regression over sampled token counts). */
typedef struct hk_line {
    double slope, offset;
} hk_line;

/* Least-squares line through `count` >= 2 samples (n[i], t[i]); *r2 (may be NULL) receives the
 * coefficient of determination.  HK_ERR_SHAPE when all n[i] are equal. */
int hk_fit_line(const double *n, const double *t, int32_t count, hk_line *line, double *r2);

/* Parameters of Algorithm 1 (the allocation of host memory to checkpoint and KV blocks). */
typedef struct hk_alloc_params {
    double T_load_w;       /* weight load latency of one decoder block */
    hk_line T_kv_gen;      /* KV generation (recompute) latency of n checkpoint blocks; slope > 0 */
    hk_line T_load_kv;     /* load latency of n KV blocks from the host; slope > 0 */
    double n_act_gpu;      /* #ACT_GPU: checkpoint blocks resident in GPU memory */
    double M_host;         /* total capacity of host memory */
    double S_weight;       /* total size of the weight parameters */
    double S_kv;           /* size of a KV block; a checkpoint block is half of it */
} hk_alloc_params;

typedef struct hk_alloc_result {
    int64_t act_init, kv_init;       /* step 1 */
    int64_t act_remain, kv_remain;   /* step 2 */
    int64_t act_host, kv_host;       /* #ACT_Host = act_init + act_remain, #KV_Host = kv_init + kv_remain */
} hk_alloc_result;

/*
 * Algorithm 1.  Step 1: T_budget = T_load_w - T_kv_gen(#ACT_GPU); if it is not negative, ACT_init is the
 * block count whose regeneration takes T_budget, otherwise KV_init is the block count whose load takes
 * -T_budget.  Step 2: the host memory left after the weights and step 1 is split into checkpoint and KV
 * blocks that fill it exactly and take equal time (T_kv_gen(#ACT) = T_load_kv(#KV)); a negative
 * solution of that 2 x 2 system is replaced by zero and the memory goes to the other kind.
 */
int hk_host_block_allocation(const hk_alloc_params *params, hk_alloc_result *result);

enum { HK_BLOCK_KV = 0, HK_BLOCK_ACT = 1 };

/*
 * Eq. 11: a request keeps #ACT_req : #KV_req = #ACT_Host : #KV_Host.  Returns the type (HK_BLOCK_ACT or
 * HK_BLOCK_KV) of the next block of a request that holds n_act checkpoint and n_kv KV blocks: the
 * one that leaves its checkpoint share nearest the host share (ties: the checkpoint block).  With the
 * paper's example, host ratio 3:1 and five checkpoint plus two KV blocks, the answer is a checkpoint
 * block.  Negative counts or an all-zero host ratio return HK_ERR_SHAPE.
 */
int hk_next_block_type(int64_t n_act, int64_t n_kv, int64_t act_host, int64_t kv_host);

/*
 * The bookkeeping of one decode step of a paged cache, on the DEVICE (Sec. 4.1; Eq. 11 with the arithmetic of
 * hk_next_block_type): every active request takes one more token.  A request whose last block is full (or that has
 * no block yet) opens logical block seq_len / block_tokens: of the kind that keeps its own #ACT : #KV nearest
 * act_host : kv_host (counted over its table row), with the next free physical block of that pool, handed out in
 * request order; its table entry is written (KV block id, or ~id for an ACT block).  Then seq_len[r] += 1 and
 * cu_tokens becomes the prefix sums of the new lengths.  After this call hk_qkv_current_paged finds the row of
 * every input token, and the attention calls find the new lengths; none of it touches the host, so all of them can
 * sit in one captured graph.
 *   block_table [B, max_blocks] int32, seq_len [B] int32, cu_tokens [B + 1] int64: device, read and written
 *   counters    [4] int32, device, read and written: [0] KV blocks in use, [1] ACT blocks in use (the next free
 *               block of a pool is its count; the caller frees by rebuilding tables and counts), [2] running
 *               count of requests that could not grow, [3] unused
 *   active      [B] int32, device, or NULL: nonzero = the request takes a token (NULL: all do)
 *   grew        [B] int32, device, or NULL; written: 1 = the request took its token in this call, 0 = it did not
 *               (inactive, or it could not grow).  It is the store_mask of the hk_qkv_current_paged call that follows.
 * A request cannot grow, keeps its length and is counted in counters[2], when its table row is full or the pool of
 * the kind it is due has no free block (the other pool is not tried: the ratio is the caller's memory plan).
 * B <= 65535.  Host checks: HK_ERR_SHAPE (sizes, block_tokens not a power of two in 16 .. 1024, a negative or
 * all-zero ratio), HK_ERR_NULL, HK_ERR_ALIGN.  B == 0 is a successful no-op.
 */
int hk_paged_append(int32_t *block_table, int32_t *seq_len, int64_t *cu_tokens, int32_t *counters, const int32_t *active,
                    int32_t *grew, int32_t B, int32_t max_blocks, int32_t block_tokens, int32_t P_kv, int32_t P_act,
                    int64_t act_host, int64_t kv_host, void *stream);

/*
 * Eq. 12 and 13 for one mini-batch: *balance = T_kv_gen(#ACT_mb) / T_load_kv(#KV_mb) and
 * *cost = F_b = max(balance, 1 / balance).  Both times must be positive.
 */
int hk_minibatch_balance(const hk_line *T_kv_gen, const hk_line *T_load_kv, double n_act_mb, double n_kv_mb,
                         double *balance, double *cost);

/* Human-readable name of a status code (static storage, never NULL). */
const char *hk_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* HYBRIDKV_H */
