"""TEST INFRASTRUCTURE -- NOT PART OF THE PRODUCT PATH.

The hybrid-cache decode step on a paged cache (Sec. 4.1, 4.2.1), stated plainly: for every request,
walk its block table, take the K/V rows of a KV block from the KV pool and regenerate the K/V rows of
an ACT block from its checkpoints (Sec. 3.3, Eq. 7, through the routines of hybridkv_oracle), join
them in logical order (Eq. 3), cut to the request's length and attend (Eq. 4).  Requests are handled
one by one; nothing is batched, tiled or reordered.  It imports nothing from the GPU package.

Pin (tests/test_paged.py): scattering a contiguous hybrid context into randomly numbered blocks and
walking the table must give what hybridkv_oracle.hybrid_decode_attn (itself pinned) gives on the
contiguous context, for any block size and any interleaving of KV and ACT blocks; plus hand-built
tables (single block, partly filled last block, empty request).

paged_append (the bookkeeping of a decode step, Eq. 11) is pinned by the worked 3:1 example of Sec. 4.3, by the
ratio every request keeps over a long run, and by the uniqueness and bounds of the blocks it hands out.
"""
import numpy as np

from . import hybridkv_oracle as ho


def paged_decode_attn(q, K_pool, V_pool, act_pool, block_table, seq_len, block_tokens,
                      gamma, beta, Wkv, bkv, n_heads, eps=1e-5, scale=None, precision="f64"):
    """q [B,H,dh]; K_pool,V_pool [P_kv,H,blk,dh]; act_pool [P_act,blk,d]; block_table [B,max_blocks]
    (entry >= 0: KV block; entry < 0: ACT block ~entry); seq_len [B].  Returns out [B,H,dh]; the
    output of a request without tokens is zero."""
    q = np.asarray(q, dtype=np.float64)
    B, H, dh = q.shape
    d = H * dh
    out = np.zeros((B, H, dh), dtype=np.float64)
    for r in range(B):
        n = int(seq_len[r])
        if n == 0:
            continue
        Ks, Vs = [], []
        for i in range((n + block_tokens - 1) // block_tokens):
            e = int(block_table[r, i])
            if e >= 0:
                Ks.append(np.asarray(K_pool[e], dtype=np.float64))
                Vs.append(np.asarray(V_pool[e], dtype=np.float64))
            else:
                k, v = ho.regen_kv(np.asarray(act_pool[~e], dtype=np.float64)[None], gamma, beta, Wkv, bkv,
                                   n_heads, eps, precision)
                Ks.append(k[0])
                Vs.append(v[0])
        K = np.concatenate(Ks, axis=1)[:, :n]            # [H, tokens, dh]
        V = np.concatenate(Vs, axis=1)[:, :n]
        out[r] = ho.decode_attention(q[r:r + 1], K[None], V[None], scale, precision=precision)[0]
    return out


def paged_append(block_table, seq_len, counters, active, block_tokens, P_kv, P_act, act_host, kv_host, with_grew=False):
    """One decode step of the paged cache's bookkeeping (Sec. 4.1; Eq. 11), request by request in order: every
    active request takes one more token; a request whose last block is full opens a new logical block of the kind
    ``policy_oracle.next_block_type`` gives for its own block counts, with the next free block of that pool
    (``counters[0]`` KV blocks and ``counters[1]`` ACT blocks are in use); a request whose table row is full or
    whose pool is exhausted keeps its length and is counted in ``counters[2]``.  Works on copies; returns
    ``(block_table, seq_len, cu_tokens, counters)``, with ``with_grew`` also which requests took their token."""
    from oracle import policy_oracle as po
    table = np.array(block_table, dtype=np.int32, copy=True)
    lens = np.array(seq_len, dtype=np.int32, copy=True)
    cnt = [int(c) for c in counters]
    B, max_blocks = table.shape
    grew = np.zeros(B, dtype=np.int32)
    for b in range(B):
        if active is not None and not active[b]:
            continue
        n = max(int(lens[b]), 0)
        if n % block_tokens == 0:
            i = n // block_tokens
            if i >= max_blocks:
                cnt[2] += 1
                continue
            n_act = int((table[b, :i] < 0).sum())
            kind = po.next_block_type(n_act, i - n_act, act_host, kv_host)
            if kind == "ACT":
                if cnt[1] >= P_act:
                    cnt[2] += 1
                    continue
                table[b, i] = ~cnt[1]
                cnt[1] += 1
            else:
                if cnt[0] >= P_kv:
                    cnt[2] += 1
                    continue
                table[b, i] = cnt[0]
                cnt[0] += 1
        lens[b] = n + 1
        grew[b] = 1
    cu = np.concatenate([[0], np.cumsum(lens.astype(np.int64))]).astype(np.int64)
    res = (table, lens, cu, np.asarray(cnt, dtype=np.int32))
    return res + (grew,) if with_grew else res
