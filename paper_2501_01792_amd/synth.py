"""Seeded synthetic OPT-shaped inputs for the hybrid-cache decode step.

This module only draws random tensors; it holds none of the method's
arithmetic and imports neither the GPU binding nor the CPU oracle, so both
sides can be fed the same fp16 bits from it.

The paper evaluates on OPT-6.7B/13B/30B/66B in fp16 with synthetic request
batches (batch size x prompt length; Sec. 5.1).  Trained weights are not
available here, so every tensor is a seeded draw with the shape of one decoder
layer of those models:

    act  [B, L_act, d]   ~ N(0, 1)             activation checkpoints
    Wkv  [2d, d]         ~ N(0, 0.02)          fused K/V projection
    bkv  [2d]            ~ N(0, 0.01)
    ln_w [d]             ~ 1 + N(0, 0.02)
    ln_b [d]             ~ N(0, 0.02)
    q    [B, H, dh]      ~ N(0, 0.02*sqrt(d))  the scale a projected vector has
    K_cache, V_cache [B, H, L_kv, dh] ~ N(0, 0.02*sqrt(d))  (same moments as
                         regenerated K/V; the step is defined for any cache content)

all rounded once to fp16.  Layer parameters come from one PCG64 stream keyed by
(seed, 0); everything that belongs to sequence ``b`` comes from a stream keyed
by (seed, 1 + tensor id, b), so any subset of sequences can be drawn alone and
has the same values as in the full batch.
"""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor

import numpy as np


@dataclasses.dataclass(frozen=True)
class LayerConfig:
    name: str
    d: int
    n_heads: int
    B: int
    L: int
    ratio: float          # fraction of the L context tokens held as cached KV
    seed: int

    @property
    def head_dim(self) -> int:
        return self.d // self.n_heads

    @property
    def L_kv(self) -> int:
        return int(round(self.ratio * self.L))

    @property
    def L_act(self) -> int:
        return self.L - self.L_kv

    @property
    def M(self) -> int:
        """Rows of the regeneration GEMM."""
        return self.B * self.L_act

    def with_ratio(self, ratio: float) -> "LayerConfig":
        return dataclasses.replace(self, ratio=ratio, name="%s@r%g" % (self.name.split("@")[0], ratio))


#: The workloads of the benchmark contract, in its order.
CONFIGS = {
    "tiny":    LayerConfig("tiny",    768,  12, 4,   256,  0.5,  0),
    "opt6.7b": LayerConfig("opt6.7b", 4096, 32, 32,  1024, 0.5,  1),
    "opt13b":  LayerConfig("opt13b",  5120, 40, 64,  2048, 0.25, 2),
    "opt30b":  LayerConfig("opt30b",  7168, 56, 128, 1024, 0.0,  3),
    "opt66b":  LayerConfig("opt66b",  9216, 72, 64,  4096, 0.0,  4),
}
SWEEP_RATIOS = (0.0, 0.25, 0.5, 0.75, 1.0)

_T_ACT, _T_Q, _T_KC, _T_VC = 1, 2, 3, 4


def _rng(*key):
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence(list(key))))


def _normal_f16(rng, shape, mean=0.0, std=1.0):
    x = rng.standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    if mean != 0.0:
        x += np.float32(mean)
    return x.astype(np.float16)


def make_params(cfg: LayerConfig) -> dict:
    """Layer parameters ``ln_w, ln_b [d]``, ``Wkv [2d, d]``, ``bkv [2d]`` as fp16 numpy arrays."""
    rng = _rng(cfg.seed, 0)
    d = cfg.d
    Wkv = _normal_f16(rng, (2 * d, d), std=0.02)
    bkv = _normal_f16(rng, (2 * d,), std=0.01)
    ln_w = _normal_f16(rng, (d,), mean=1.0, std=0.02)
    ln_b = _normal_f16(rng, (d,), std=0.02)
    return {"ln_w": ln_w, "ln_b": ln_b, "Wkv": Wkv, "bkv": bkv}


def make_current_token(cfg: LayerConfig) -> dict:
    """Inputs of the current-token QKV generation: ``x_cur [B, d] ~ N(0, 1)`` (a layer input, like the
    checkpoints), ``Wq [d, d] ~ N(0, 0.02)``, ``bq [d] ~ N(0, 0.01)``; their own stream keyed (seed, 9)."""
    rng = _rng(cfg.seed, 9)
    d = cfg.d
    return {"x_cur": _normal_f16(rng, (cfg.B, d)), "Wq": _normal_f16(rng, (d, d), std=0.02),
            "bq": _normal_f16(rng, (d,), std=0.01)}


def make_sequence(cfg: LayerConfig, b: int) -> dict:
    """Per-sequence tensors of sequence ``b``: ``act [L_act, d]``, ``q [H, dh]``,
    ``K_cache, V_cache [H, L_kv, dh]`` (fp16)."""
    H, dh, d = cfg.n_heads, cfg.head_dim, cfg.d
    kv_std = 0.02 * float(np.sqrt(d))
    return {
        "act": _normal_f16(_rng(cfg.seed, _T_ACT, b), (cfg.L_act, d)),
        "q": _normal_f16(_rng(cfg.seed, _T_Q, b), (H, dh), std=kv_std),
        "K_cache": _normal_f16(_rng(cfg.seed, _T_KC, b), (H, cfg.L_kv, dh), std=kv_std),
        "V_cache": _normal_f16(_rng(cfg.seed, _T_VC, b), (H, cfg.L_kv, dh), std=kv_std),
    }


def make_batch(cfg: LayerConfig, sequences=None, threads: int = 8) -> dict:
    """Stack ``make_sequence`` over ``sequences`` (default: all ``cfg.B``) and add the
    layer parameters.  Returns fp16 numpy arrays ``q [n,H,dh]``, ``act [n,L_act,d]``,
    ``K_cache, V_cache [n,H,L_kv,dh]``, ``ln_w, ln_b, Wkv, bkv``."""
    seqs = list(range(cfg.B)) if sequences is None else list(sequences)
    n = len(seqs)
    H, dh, d = cfg.n_heads, cfg.head_dim, cfg.d
    out = {
        "q": np.empty((n, H, dh), np.float16),
        "act": np.empty((n, cfg.L_act, d), np.float16),
        "K_cache": np.empty((n, H, cfg.L_kv, dh), np.float16),
        "V_cache": np.empty((n, H, cfg.L_kv, dh), np.float16),
    }

    def fill(i):
        s = make_sequence(cfg, seqs[i])
        for k in ("q", "act", "K_cache", "V_cache"):
            out[k][i] = s[k]

    if threads > 1 and n > 1:
        with ThreadPoolExecutor(max_workers=min(threads, n)) as ex:
            list(ex.map(fill, range(n)))
    else:
        for i in range(n):
            fill(i)
    out.update(make_params(cfg))
    return out


def scatter_into_blocks(cfg: LayerConfig, batch: dict, seq_len, block_tokens: int, act_fraction: float, seed: int) -> dict:
    """Lays a contiguous hybrid context out as a paged cache: request b keeps ``seq_len[b]`` tokens; each of
    its logical blocks becomes an ACT block with probability ``act_fraction`` (one number, or one per request)
    and a KV block otherwise;
    physical block numbers are a random permutation of each pool (with spare, never referenced blocks).
    ``batch`` needs ``act_full [B, L, d]`` (the layer inputs of every token) and ``K_full, V_full [B, H, L, dh]``
    (their K/V rows).  Data movement only: no arithmetic of the method."""
    rng = _rng(cfg.seed, 77, seed)
    B, H, dh, d, bt = cfg.B, cfg.n_heads, cfg.head_dim, cfg.d, block_tokens
    n_blocks = [(int(n) + bt - 1) // bt for n in seq_len]
    max_blocks = max(max(n_blocks), 1)
    frac = np.broadcast_to(np.asarray(act_fraction, dtype=np.float64), (B,))
    kinds = [rng.random(nb) < frac[b] for b, nb in enumerate(n_blocks)]
    n_act = int(sum(int(k.sum()) for k in kinds))
    n_kv = int(sum(n_blocks)) - n_act
    P_act, P_kv = n_act + 2, n_kv + 3
    act_ids = rng.permutation(n_act)                     # ACT blocks in use are 0 .. n_act - 1
    kv_ids = rng.permutation(P_kv)[:n_kv]
    K_pool = _normal_f16(rng, (P_kv, H, bt, dh), std=3.0)   # spare blocks and unused rows hold unrelated numbers
    V_pool = _normal_f16(rng, (P_kv, H, bt, dh), std=3.0)
    act_pool = _normal_f16(rng, (P_act, bt, d), std=1.0)
    table = np.full((B, max_blocks), 0x7fffffff, dtype=np.int32)   # never read beyond a request's blocks
    ia = ik = 0
    for b in range(B):
        for i in range(n_blocks[b]):
            t0, t1 = i * bt, min((i + 1) * bt, int(seq_len[b]))
            if kinds[b][i]:
                pb = int(act_ids[ia]); ia += 1
                act_pool[pb, :t1 - t0] = batch["act_full"][b, t0:t1]
                table[b, i] = ~pb
            else:
                pb = int(kv_ids[ik]); ik += 1
                K_pool[pb, :, :t1 - t0] = batch["K_full"][b, :, t0:t1]
                V_pool[pb, :, :t1 - t0] = batch["V_full"][b, :, t0:t1]
                table[b, i] = pb
    return {"K_pool": K_pool, "V_pool": V_pool, "act_pool": act_pool, "block_table": table,
            "seq_len": np.asarray(seq_len, dtype=np.int32), "n_act_used": n_act, "kinds": kinds}
