// One decode step of the paged cache's bookkeeping, on the device (Sec. 4.1 block tables, Sec. 4.3 Eq. 11): every
// active request takes one more token; a request whose last block is full opens a new logical block, of the kind
// that keeps its own #ACT : #KV nearest the host ratio (the rule of hk_next_block_type, in the same integer
// arithmetic), with the next free physical block of that pool; lengths and their prefix sums are updated.  Nothing
// here touches the host, so the step can sit in a captured graph between hk_qkv_current_paged calls.
//
// One workgroup walks the requests 256 at a time.  Physical blocks are handed out in request order (a block-wide
// exclusive scan of the requests that need one of each kind), so the result does not depend on scheduling.  A
// request that cannot grow (its table row is full, or the pool of the kind it is due has no free block) keeps its
// length and is counted.
#include "hk_internal.h"

namespace hk {
namespace {

constexpr int kThreads = 256;

// exclusive scan of one flag per thread over the workgroup; returns the thread's rank, *total the number of flags
__device__ __forceinline__ int block_rank(bool flag, int *scratch, int *total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const unsigned long long mask = __ballot(flag);
    const int in_wave = __popcll(mask & ((1ull << lane) - 1ull));
    if (lane == 0) scratch[wave] = __popcll(mask);
    __syncthreads();
    int before = 0, all = 0;
#pragma unroll
    for (int w = 0; w < kThreads / 64; ++w) {
        const int c = scratch[w];
        if (w < wave) before += c;
        all += c;
    }
    __syncthreads();                                       // scratch is reused by the next call
    *total = all;
    return before + in_wave;
}

__global__ __launch_bounds__(kThreads) void paged_append_kernel(int32_t *__restrict__ table, int32_t *__restrict__ seq_len,
                                                                int64_t *__restrict__ cu, int32_t *__restrict__ counters,
                                                                const int32_t *__restrict__ active, int32_t *__restrict__ grew,
                                                                int B, int max_blocks,
                                                                int blk_log2, int P_kv, int P_act, int64_t act_host, int64_t kv_host)
{
    __shared__ int scratch[kThreads / 64];
    __shared__ long long wave_sum[kThreads / 64];
    int kv_used = counters[0], act_used = counters[1], failed = 0;   // every thread keeps the same running copies
    long long carry = 0;                                             // tokens of the requests before this chunk
    const int bt_mask = (1 << blk_log2) - 1;
    for (int base = 0; base < B; base += kThreads) {
        const int b = base + (int)threadIdx.x;
        const bool in = b < B;
        int len = in ? seq_len[b] : 0;
        if (len < 0) len = 0;
        const bool grows = in && (active == nullptr || active[b] != 0);
        const bool opens = grows && (len & bt_mask) == 0;            // the last block is full (or there is none yet)
        const int idx = len >> blk_log2;                             // logical block the new token falls into
        bool want_act = false, stuck = false;
        if (opens) {
            if (idx >= max_blocks) {
                stuck = true;
            } else {
                // the kinds of the blocks the request holds; the loads of a pass do not depend on each other
                const int32_t *row = table + (int64_t)b * max_blocks;
                int acts = 0, i = 0;
                for (; i + 8 <= idx; i += 8) {
                    int32_t e[8];
#pragma unroll
                    for (int j = 0; j < 8; ++j) e[j] = row[i + j];
#pragma unroll
                    for (int j = 0; j < 8; ++j) acts += e[j] < 0;
                }
                for (; i < idx; ++i) acts += row[i] < 0;
                const long long n_act = acts, n_kv = idx - acts;
                if (kv_host == 0) want_act = true;
                else if (act_host == 0) want_act = false;
                else {
                    // the checkpoint share after the allocation nearest act_host / (act_host + kv_host); ties: checkpoint
                    const long long T = act_host + kv_host, n1 = n_act + n_kv + 1;
                    long long da = (n_act + 1) * T - act_host * n1, dk = n_act * T - act_host * n1;
                    if (da < 0) da = -da;
                    if (dk < 0) dk = -dk;
                    want_act = da <= dk;
                }
            }
        }
        int n_a, n_k;
        const int rank_a = block_rank(opens && !stuck && want_act, scratch, &n_a);
        const int rank_k = block_rank(opens && !stuck && !want_act, scratch, &n_k);
        bool ok = grows && !stuck;
        if (opens && !stuck) {
            const int id = want_act ? act_used + rank_a : kv_used + rank_k;
            if (id < (want_act ? P_act : P_kv)) table[(int64_t)b * max_blocks + idx] = want_act ? ~id : id;
            else ok = false;                                         // that pool is exhausted
        }
        const int new_len = ok ? len + 1 : len;
        if (in && ok) seq_len[b] = new_len;
        if (in && grew) grew[b] = ok ? 1 : 0;                        // whether the request holds a new token after this call
        int n_fail;
        block_rank(grows && !ok, scratch, &n_fail);
        failed += n_fail;
        act_used = act_used + n_a < P_act ? act_used + n_a : P_act;  // requests past the end of a pool got nothing
        kv_used = kv_used + n_k < P_kv ? kv_used + n_k : P_kv;
        // prefix sums of the lengths: wavefront scan, then across the four wavefronts
        long long v = in ? new_len : 0;
        const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const long long up = __shfl_up(v, off, 64);
            if (lane >= off) v += up;
        }
        if (lane == 63) wave_sum[wave] = v;
        __syncthreads();
        long long before = 0, all = 0;
#pragma unroll
        for (int w = 0; w < kThreads / 64; ++w) {
            if (w < wave) before += wave_sum[w];
            all += wave_sum[w];
        }
        if (in) cu[b + 1] = carry + before + v;
        carry += all;
        __syncthreads();                                             // wave_sum is reused by the next chunk
    }
    if (threadIdx.x == 0) {
        cu[0] = 0;
        counters[0] = kv_used;
        counters[1] = act_used;
        counters[2] += failed;
    }
}

}  // namespace

hipError_t launch_paged_append(const PagedAppendArgs &a, hipStream_t s)
{
    if (a.B <= 0) return hipSuccess;
    if (a.block_tokens < 16 || (a.block_tokens & (a.block_tokens - 1)) != 0 || a.max_blocks <= 0 || a.P_kv < 0 || a.P_act < 0 ||
        a.act_host < 0 || a.kv_host < 0 || a.act_host + a.kv_host <= 0 || a.act_host > (1LL << 31) || a.kv_host > (1LL << 31))
        return hipErrorInvalidValue;
    int blk_log2 = 0;
    while ((1 << blk_log2) < a.block_tokens) ++blk_log2;
    hipLaunchKernelGGL(paged_append_kernel, dim3(1), dim3(kThreads), 0, s, a.block_table, a.seq_len, a.cu_tokens, a.counters,
                       a.active, a.grew, a.B, a.max_blocks, blk_log2, a.P_kv, a.P_act, a.act_host, a.kv_host);
    return hipGetLastError();
}

}  // namespace hk
