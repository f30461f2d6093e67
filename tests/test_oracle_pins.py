"""Pins of the CPU oracle against things other than itself.

The paper prints no worked numerical example of the step, so the oracle is
pinned by: a hand-worked two-token case (tests/golden/two_token_case.txt),
closed forms and invariants of LayerNorm / Eq. 7 / Eq. 4, brute force written
as Python loops straight from the definitions, torch's CPU library routines,
and the method's own exactness claim (Sec. 3.3: regenerating K/V from the
checkpoints gives the same result as caching them), i.e. ratio invariance.
Each pin is chosen so that a plausible slip (dropped term, wrong sign or index,
transposed operand, wrong head split) fails at least one of them.
"""
import math
import os

import numpy as np
import pytest
import torch

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read_fixture(name):
    vals = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *rest = line.split()
            vals[key] = np.array([float(v) for v in rest], dtype=np.float64)
    return vals


def _rand(shape, seed, scale=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * scale


# ---------------------------------------------------------------- whole step, by hand
@pytest.mark.parametrize("precision,tol", [("f64", 1e-14), ("f32", 1e-6)])
def test_two_token_case_by_hand(oracle, precision, tol):
    fx = _read_fixture("two_token_case.txt")
    d, H = int(fx["d"][0]), int(fx["n_heads"][0])
    q = (fx["q_dir"] * math.log(3.0) / math.sqrt(2.0)).reshape(1, H, d)
    act = fx["act"].reshape(1, 2, d)
    Wkv, bkv = fx["Wkv"].reshape(2 * d, d), fx["bkv"]
    K_exp, V_exp = fx["K"].reshape(1, 1, 2, d), fx["V"].reshape(1, 1, 2, d)
    args = dict(gamma=fx["ln_w"], beta=fx["ln_b"], Wkv=Wkv, bkv=bkv, n_heads=H,
                eps=float(fx["eps"][0]), precision=precision)
    # ratio 0: both tokens are checkpoints
    out, K, V = oracle.hybrid_decode_attn(q, None, None, act, **args)
    np.testing.assert_allclose(K, K_exp, atol=tol)
    np.testing.assert_allclose(V, V_exp, atol=tol)
    np.testing.assert_allclose(out.ravel(), fx["out"], atol=tol)
    # ratio 1/2: token 1 arrives as a cached K/V row, token 2 as a checkpoint
    out2, K2, V2 = oracle.hybrid_decode_attn(q, K_exp[:, :, :1], V_exp[:, :, :1], act[:, 1:], **args)
    np.testing.assert_allclose(out2.ravel(), fx["out"], atol=tol)
    np.testing.assert_allclose(K2, K_exp, atol=tol)
    # ratio 1: both cached
    out3, _, _ = oracle.hybrid_decode_attn(q, K_exp, V_exp, None, **args)
    np.testing.assert_allclose(out3.ravel(), fx["out"], atol=tol)
    # the softmax row itself
    _, p = oracle.decode_attention(q, K_exp, V_exp, return_probs=True, precision=precision)
    np.testing.assert_allclose(p.ravel(), fx["probs"], atol=tol)


def test_two_token_case_with_eps_closed_form(oracle):
    """Same case with the usual eps = 1e-5: xhat = +-c, c = (1+eps)^-1/2, and
    out = c * tanh(c * ln(3)/2) * (1, -1)."""
    fx = _read_fixture("two_token_case.txt")
    eps = 1e-5
    c = 1.0 / math.sqrt(1.0 + eps)
    q = (fx["q_dir"] * math.log(3.0) / math.sqrt(2.0)).reshape(1, 1, 2)
    out, K, _ = oracle.hybrid_decode_attn(q, None, None, fx["act"].reshape(1, 2, 2), fx["ln_w"], fx["ln_b"],
                                          fx["Wkv"].reshape(4, 2), fx["bkv"], 1, eps=eps)
    e = c * math.tanh(c * math.log(3.0) / 2.0)
    np.testing.assert_allclose(out.ravel(), [e, -e], atol=1e-14)
    np.testing.assert_allclose(K.ravel(), [c, -c, -c, c], atol=1e-14)


# ---------------------------------------------------------------- LayerNorm
def test_layernorm_matches_torch_library(oracle):
    x = _rand((37, 96), 1, 3.0) + 0.7
    g, b = 1 + _rand(96, 2, 0.3), _rand(96, 3, 0.3)
    ref = torch.nn.functional.layer_norm(torch.from_numpy(x), (96,), torch.from_numpy(g),
                                         torch.from_numpy(b), eps=1e-5).numpy()
    np.testing.assert_allclose(oracle.layernorm(x, g, b, 1e-5), ref, rtol=0, atol=1e-12)
    ref32 = torch.nn.functional.layer_norm(torch.from_numpy(x).float(), (96,), torch.from_numpy(g).float(),
                                           torch.from_numpy(b).float(), eps=1e-5).numpy()
    np.testing.assert_allclose(oracle.layernorm(x, g, b, 1e-5, precision="f32"), ref32, atol=5e-6)


def test_layernorm_moments_and_invariances(oracle):
    d = 64
    x = _rand((11, d), 4, 2.0) + 5.0
    one, zero = np.ones(d), np.zeros(d)
    eps = 1e-5
    y = oracle.layernorm(x, one, zero, eps)
    np.testing.assert_allclose(y.mean(axis=1), 0, atol=1e-14)
    var = x.var(axis=1)                              # biased variance
    np.testing.assert_allclose((y * y).mean(axis=1), var / (var + eps), rtol=1e-13)
    np.testing.assert_allclose(oracle.layernorm(x + 123.25, one, zero, eps), y, atol=1e-12)    # shift
    np.testing.assert_allclose(oracle.layernorm(x * 8.0, one, zero, eps), y, atol=1e-5)        # scale (eps-limited)
    np.testing.assert_allclose(oracle.layernorm(-x, one, zero, eps), -y, atol=1e-14)           # odd
    g, b = 1 + _rand(d, 5, 0.5), _rand(d, 6, 0.5)
    np.testing.assert_allclose(oracle.layernorm(x, g, b, eps), y * g + b, atol=1e-14)          # affine per column
    # eps sits inside the square root: a constant row maps to beta, and a huge eps flattens the row
    np.testing.assert_allclose(oracle.layernorm(np.full((1, d), 3.0), g, b, eps), b[None], atol=1e-14)
    np.testing.assert_allclose(oracle.layernorm(x, one, zero, 1e12), (x - x.mean(1, keepdims=True)) / 1e6, rtol=1e-9, atol=1e-12)


# ---------------------------------------------------------------- Eq. 7
def test_projection_brute_force_and_library(oracle):
    M, d = 5, 6
    xh, W, b = _rand((M, d), 7), _rand((2 * d, d), 8), _rand(2 * d, 9)
    got = oracle.kv_projection(xh, W, b)
    # Eq. 7 spelled out: [K V] = A x [W_K W_V], W_K[j, n] = Wkv[n, j]
    W_K, W_V = W[:d].T, W[d:].T
    for r in range(M):
        for n in range(d):
            k = sum(xh[r, j] * W_K[j, n] for j in range(d)) + b[n]
            v = sum(xh[r, j] * W_V[j, n] for j in range(d)) + b[d + n]
            assert abs(got[r, n] - k) < 1e-13 and abs(got[r, d + n] - v) < 1e-13
    ref = torch.nn.functional.linear(torch.from_numpy(xh), torch.from_numpy(W), torch.from_numpy(b)).numpy()
    np.testing.assert_allclose(got, ref, atol=1e-13)
    np.testing.assert_allclose(got, np.concatenate([xh @ W_K, xh @ W_V], axis=1) + b, atol=1e-13)


def test_projection_identity_and_linearity(oracle):
    M, d = 4, 8
    xh = _rand((M, d), 10)
    eye2 = np.concatenate([np.eye(d), np.eye(d)], axis=0)
    np.testing.assert_allclose(oracle.kv_projection(xh, eye2, np.zeros(2 * d)), np.concatenate([xh, xh], 1), atol=0)
    W1, W2, b1, b2 = _rand((2 * d, d), 11), _rand((2 * d, d), 12), _rand(2 * d, 13), _rand(2 * d, 14)
    lhs = oracle.kv_projection(xh, 2 * W1 - 3 * W2, 2 * b1 - 3 * b2)
    rhs = 2 * oracle.kv_projection(xh, W1, b1) - 3 * oracle.kv_projection(xh, W2, b2)
    np.testing.assert_allclose(lhs, rhs, atol=1e-12)
    # a single 1 at Wkv[n, j] routes input feature j to output feature n (not the other way round)
    W = np.zeros((2 * d, d)); W[3, 5] = 1.0; W[d + 1, 2] = 1.0
    out = oracle.kv_projection(xh, W, np.zeros(2 * d))
    exp = np.zeros((M, 2 * d)); exp[:, 3] = xh[:, 5]; exp[:, d + 1] = xh[:, 2]
    np.testing.assert_allclose(out, exp, atol=0)


@pytest.mark.parametrize("H", [1, 2, 4])
def test_regen_kv_head_split_brute_force(oracle, H):
    B, L, d = 2, 3, 8
    dh = d // H
    act = _rand((B, L, d), 15, 2.0) + 0.3
    g, be = 1 + _rand(d, 16, 0.2), _rand(d, 17, 0.2)
    W, bias = _rand((2 * d, d), 18, 0.3), _rand(2 * d, 19, 0.1)
    eps = 1e-5
    K, V = oracle.regen_kv(act, g, be, W, bias, H, eps)
    assert K.shape == (B, H, L, dh)
    for b in range(B):
        for t in range(L):
            x = act[b, t]
            mu = sum(x) / d
            var = sum((xi - mu) ** 2 for xi in x) / d
            xh = [(x[j] - mu) / math.sqrt(var + eps) * g[j] + be[j] for j in range(d)]
            for n in range(d):
                k = sum(xh[j] * W[n, j] for j in range(d)) + bias[n]
                v = sum(xh[j] * W[d + n, j] for j in range(d)) + bias[d + n]
                assert abs(K[b, n // dh, t, n % dh] - k) < 1e-12
                assert abs(V[b, n // dh, t, n % dh] - v) < 1e-12


# ---------------------------------------------------------------- Eq. 4
def test_attention_matches_torch_and_unstabilised_softmax(oracle):
    B, H, L, dh = 2, 3, 17, 8
    q, K, V = _rand((B, H, dh), 20), _rand((B, H, L, dh), 21), _rand((B, H, L, dh), 22)
    out, p = oracle.decode_attention(q, K, V, return_probs=True)
    np.testing.assert_allclose(p.sum(-1), 1.0, atol=1e-14)
    tq, tK, tV = map(torch.from_numpy, (q, K, V))
    s = torch.einsum("bhd,bhld->bhl", tq, tK) * dh ** -0.5
    tp = torch.softmax(s, dim=-1)
    np.testing.assert_allclose(p, tp.numpy(), atol=1e-14)
    np.testing.assert_allclose(out, torch.einsum("bhl,bhld->bhd", tp, tV).numpy(), atol=1e-13)
    # definition without the max subtraction, as Python loops
    for b in range(B):
        for h in range(H):
            e = [math.exp(sum(q[b, h, i] * K[b, h, t, i] for i in range(dh)) / math.sqrt(dh)) for t in range(L)]
            Z = sum(e)
            for i in range(dh):
                o = sum(e[t] / Z * V[b, h, t, i] for t in range(L))
                assert abs(out[b, h, i] - o) < 1e-13


def test_attention_special_cases(oracle):
    B, H, L, dh = 1, 2, 9, 4
    q, K, V = _rand((B, H, dh), 23), _rand((B, H, L, dh), 24), _rand((B, H, L, dh), 25)
    # q = 0: uniform weights -> mean of the value rows
    np.testing.assert_allclose(oracle.decode_attention(np.zeros_like(q), K, V), V.mean(axis=2), atol=1e-14)
    # all value rows equal -> that row, whatever the scores
    Vc = np.broadcast_to(V[:, :, :1], V.shape)
    np.testing.assert_allclose(oracle.decode_attention(q, K, Vc), V[:, :, 0], atol=1e-14)
    # one key aligned with a huge query dominates
    Kd = K.copy(); Kd[:, :, 5] = q * 1e3
    np.testing.assert_allclose(oracle.decode_attention(q * 10, Kd, V), V[:, :, 5], atol=1e-12)
    # huge scores do not overflow (max is subtracted)
    out = oracle.decode_attention(q * 1e4, K, V, precision="f32")
    assert np.isfinite(out).all()
    # adding the same vector to every key shifts all scores of a head equally: softmax unchanged
    np.testing.assert_allclose(oracle.decode_attention(q, K + _rand((B, H, 1, dh), 26), V),
                               oracle.decode_attention(q, K, V), atol=1e-13)
    # the scale multiplies the scores: scale 0 == q 0
    np.testing.assert_allclose(oracle.decode_attention(q, K, V, scale=0.0), V.mean(axis=2), atol=1e-14)
    # a single context token: out is its value row
    np.testing.assert_allclose(oracle.decode_attention(q, K[:, :, :1], V[:, :, :1]), V[:, :, 0], atol=0)
    # heads and sequences are independent: head 1 of the batch == a one-head problem
    np.testing.assert_allclose(oracle.decode_attention(q, K, V)[:, 1:], oracle.decode_attention(q[:, 1:], K[:, 1:], V[:, 1:]), atol=0)


# ---------------------------------------------------------------- the method's exactness claim
def _small_problem(seed, B=3, H=2, dh=8, L=12):
    d = H * dh
    act = _rand((B, L, d), seed, 1.5) + 0.2
    g, be = 1 + _rand(d, seed + 1, 0.1), _rand(d, seed + 2, 0.1)
    W, bias = _rand((2 * d, d), seed + 3, 0.2), _rand(2 * d, seed + 4, 0.1)
    q = _rand((B, H, dh), seed + 5)
    return act, g, be, W, bias, q, H


@pytest.mark.parametrize("precision,tol", [("f64", 1e-13), ("f32", 2e-6)])
def test_ratio_invariance(oracle, precision, tol):
    """Sec. 3.3: regeneration reproduces the KV-cache result, so the output
    cannot depend on how the context is split between the two stores."""
    act, g, be, W, bias, q, H = _small_problem(30)
    L = act.shape[1]
    Kf, Vf = oracle.regen_kv(act, g, be, W, bias, H, precision=precision)
    ref = oracle.decode_attention(q, Kf, Vf, precision=precision)
    for L_kv in (0, 3, 6, 9, L):
        Kc = Kf[:, :, :L_kv] if L_kv else None
        Vc = Vf[:, :, :L_kv] if L_kv else None
        a = act[:, L_kv:] if L_kv < L else None
        out, K2, V2 = oracle.hybrid_decode_attn(q, Kc, Vc, a, g, be, W, bias, H, precision=precision)
        np.testing.assert_allclose(out, ref, atol=tol)
        np.testing.assert_allclose(K2, Kf, atol=tol)
        np.testing.assert_allclose(V2, Vf, atol=tol)


def test_token_order_invariance(oracle):
    """Softmax attention sums over context tokens: any assignment of tokens to
    the two stores (any permutation of the context) gives the same output."""
    act, g, be, W, bias, q, H = _small_problem(40)
    L = act.shape[1]
    Kf, Vf = oracle.regen_kv(act, g, be, W, bias, H)
    ref = oracle.decode_attention(q, Kf, Vf)
    perm = np.random.default_rng(41).permutation(L)
    kv_tok, act_tok = perm[:5], perm[5:]
    out, _, _ = oracle.hybrid_decode_attn(q, Kf[:, :, kv_tok], Vf[:, :, kv_tok], act[:, act_tok], g, be, W, bias, H)
    np.testing.assert_allclose(out, ref, atol=1e-13)


def test_f32_build_agrees_with_f64(oracle):
    """Bounds the fp32 baseline's own rounding at a long reduction (d = 1024)."""
    rng = np.random.default_rng(50)
    B, H, dh, L = 2, 8, 128, 40
    d = H * dh
    act = rng.standard_normal((B, L, d)).astype(np.float16)
    g = (1 + 0.02 * rng.standard_normal(d)).astype(np.float16)
    be = (0.02 * rng.standard_normal(d)).astype(np.float16)
    W = (0.02 * rng.standard_normal((2 * d, d))).astype(np.float16)
    bias = (0.01 * rng.standard_normal(2 * d)).astype(np.float16)
    q = rng.standard_normal((B, H, dh)).astype(np.float16)
    o64, K64, _ = oracle.hybrid_decode_attn(q, None, None, act, g, be, W, bias, H)
    o32, K32, _ = oracle.hybrid_decode_attn(q, None, None, act, g, be, W, bias, H, precision="f32")
    assert np.linalg.norm(K32 - K64) / np.linalg.norm(K64) < 1e-5
    assert np.linalg.norm(o32 - o64) / np.linalg.norm(o64) < 1e-5


# ---------------------------------------------------------------- the pins do catch slips
def test_pins_detect_planted_mistakes(oracle):
    """Sanity of the pins themselves: typical slips, planted here on the CPU in a
    copy of the definition, are told apart from the oracle by the same checks."""
    x = _rand((4, 16), 60, 2.0) + 1.0
    one, zero = np.ones(16), np.zeros(16)
    y = oracle.layernorm(x, one, zero, 1e-5)
    unbiased = (x - x.mean(1, keepdims=True)) / np.sqrt(x.var(1, ddof=1, keepdims=True) + 1e-5)
    assert np.abs(unbiased - y).max() > 1e-3                       # biased vs unbiased variance
    eps_outside = (x - x.mean(1, keepdims=True)) / (np.sqrt(x.var(1, keepdims=True)) + 1e-1)
    assert np.abs(eps_outside - oracle.layernorm(x, one, zero, 1e-1)).max() > 1e-3
    xh, W, b = _rand((3, 4), 61), _rand((8, 4), 62), _rand(8, 63)
    got = oracle.kv_projection(xh, W, b)
    swapped = np.concatenate([xh @ W[4:].T, xh @ W[:4].T], 1) + b   # K and V blocks exchanged
    assert np.abs(swapped - got).max() > 1e-2
    q, K, V = _rand((1, 1, 4), 64), _rand((1, 1, 6, 4), 65), _rand((1, 1, 6, 4), 66)
    unscaled = oracle.decode_attention(q, K, V, scale=1.0)
    assert np.abs(unscaled - oracle.decode_attention(q, K, V)).max() > 1e-3   # the dh^-1/2 scale matters


# ---------------------------------------------------------------- current-token QKV generation
def test_qkv_current_brute_force_and_library(oracle):
    """q, k, v of the current token against Python loops written from Eq. 2 (+ LayerNorm, biases)
    and against torch's CPU layer_norm / linear; head split checked index by index."""
    rng = np.random.default_rng(31)
    B, d, H = 3, 12, 3
    dh = d // H
    x = rng.standard_normal((B, d)) * 2 + 0.5
    g, be = 1 + 0.1 * rng.standard_normal(d), 0.1 * rng.standard_normal(d)
    Wq, bq = rng.standard_normal((d, d)), rng.standard_normal(d)
    Wkv, bkv = rng.standard_normal((2 * d, d)), rng.standard_normal(2 * d)
    q, k, v = oracle.qkv_current(x, g, be, Wq, bq, Wkv, bkv, H, eps=1e-5)
    for b in range(B):
        mu = sum(x[b]) / d
        var = sum((x[b, j] - mu) ** 2 for j in range(d)) / d
        xh = [(x[b, j] - mu) / math.sqrt(var + 1e-5) * g[j] + be[j] for j in range(d)]
        for n in range(d):
            h, i = divmod(n, dh)
            assert abs(q[b, h, i] - (sum(xh[j] * Wq[n, j] for j in range(d)) + bq[n])) < 1e-12
            assert abs(k[b, h, i] - (sum(xh[j] * Wkv[n, j] for j in range(d)) + bkv[n])) < 1e-12
            assert abs(v[b, h, i] - (sum(xh[j] * Wkv[d + n, j] for j in range(d)) + bkv[d + n])) < 1e-12
    xt = torch.nn.functional.layer_norm(torch.from_numpy(x), (d,), torch.from_numpy(g), torch.from_numpy(be), 1e-5)
    qt = torch.nn.functional.linear(xt, torch.from_numpy(Wq), torch.from_numpy(bq)).numpy().reshape(B, H, dh)
    np.testing.assert_allclose(q, qt, atol=1e-12)


def test_current_token_joins_either_store_with_the_same_result(oracle):
    """Sec. 4.2.2: the input token's K/V take part in its own attention and the token is then kept as
    a KV entry or as a checkpoint.  Both routes must give the step the same output: appending its
    (k, v) to the cache, or appending its layer input to the checkpoints (Sec. 3.3's exactness)."""
    rng = np.random.default_rng(32)
    B, d, H, L_kv, L_act = 2, 16, 4, 3, 5
    dh = d // H
    g, be = 1 + 0.1 * rng.standard_normal(d), 0.1 * rng.standard_normal(d)
    Wq, bq = rng.standard_normal((d, d)) * 0.3, rng.standard_normal(d) * 0.1
    Wkv, bkv = rng.standard_normal((2 * d, d)) * 0.3, rng.standard_normal(2 * d) * 0.1
    x = rng.standard_normal((B, d))
    act = rng.standard_normal((B, L_act, d))
    Kc, Vc = rng.standard_normal((B, H, L_kv, dh)), rng.standard_normal((B, H, L_kv, dh))
    q, k, v = oracle.qkv_current(x, g, be, Wq, bq, Wkv, bkv, H)
    out_kv, _, _ = oracle.hybrid_decode_attn(q, np.concatenate([Kc, k[:, :, None]], axis=2),
                                             np.concatenate([Vc, v[:, :, None]], axis=2), act, g, be, Wkv, bkv, H)
    out_act, K_full, _ = oracle.hybrid_decode_attn(q, Kc, Vc, np.concatenate([act, x[:, None]], axis=1),
                                                   g, be, Wkv, bkv, H)
    np.testing.assert_allclose(out_kv, out_act, atol=1e-12)
    np.testing.assert_allclose(K_full[:, :, -1], k, atol=1e-12)      # the regenerated row of the token is its k


def test_projections_moved_across_the_sums_give_the_same_step(oracle):
    """The identity behind hk_hybrid_decode_attn_absorbed, in fp64 and with the oracle as the reference: for
    one query per head the K projection of Eq. 7 can be applied to the query and the V projection to the
    weighted sum of the checkpoint rows, LayerNorm folded in, the cached segment joined through its softmax
    maximum and denominator.  Written with plain numpy from the formulas in include/hybridkv.h; any slip in
    them (a missing mean term, a wrong head slice, the join) shows here without a GPU."""
    rng = np.random.default_rng(3)
    B, H, dh, L_kv, L_act, eps = 3, 2, 8, 13, 24, 1e-5
    d = H * dh
    q = rng.standard_normal((B, H, dh))
    Kc, Vc = rng.standard_normal((B, H, L_kv, dh)), rng.standard_normal((B, H, L_kv, dh))
    act = rng.standard_normal((B, L_act, d)) * rng.uniform(0.2, 3.0, size=(B, L_act, 1)) + rng.uniform(-5, 5, size=(B, L_act, 1))
    g, be = 1 + 0.2 * rng.standard_normal(d), 0.2 * rng.standard_normal(d)
    W, bias = rng.standard_normal((2 * d, d)) * 0.3, rng.standard_normal(2 * d) * 0.1
    ref, _, _ = oracle.hybrid_decode_attn(q, Kc, Vc, act, g, be, W, bias, H)
    Wp = W * g[None, :]                                    # gamma folded into the weights
    bp = bias + W @ be                                     # beta folded into the bias
    scale = dh ** -0.5
    out = np.empty_like(ref)
    for s in range(B):
        x = act[s]
        mean = x.mean(axis=1)
        rstd = 1.0 / np.sqrt(x.var(axis=1) + eps)
        for h in range(H):
            ks, vs = slice(h * dh, (h + 1) * dh), slice(d + h * dh, d + (h + 1) * dh)
            u = q[s, h] @ Wp[ks]                           # the query carried through the key weights  [d]
            sc_a = scale * (rstd * (x @ u - mean * u.sum()) + q[s, h] @ bp[ks])
            m_a = sc_a.max()
            p = np.exp(sc_a - m_a)
            l_a = p.sum()
            y = ((p * rstd / l_a)[:, None] * (x - mean[:, None])).sum(axis=0)      # weighted, centred row sum  [d]
            o_a = Wp[vs] @ y + bp[vs]
            sc_c = scale * (Kc[s, h] @ q[s, h])
            m_c = sc_c.max()
            pc = np.exp(sc_c - m_c)
            l_c = pc.sum()
            o_c = pc @ Vc[s, h] / l_c
            m = max(m_a, m_c)
            wa, wc = l_a * np.exp(m_a - m), l_c * np.exp(m_c - m)
            out[s, h] = (wa * o_a + wc * o_c) / (wa + wc)
    assert np.abs(out - ref).max() <= 1e-10 * max(1.0, np.abs(ref).max())
