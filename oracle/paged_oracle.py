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
