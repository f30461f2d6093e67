/*
 * TEST INFRASTRUCTURE -- NOT PART OF THE PRODUCT PATH.
 *
 * Body of the CPU oracle for the per-layer hybrid-cache decode step, written
 * once and compiled twice by hybridkv_oracle.c: with REAL = double (the
 * reference result) and with REAL = float (the "plain fp32" baseline that is
 * timed next to the GPU path).  Only tests, the smoke check and the bench's
 * cpu_baseline leg may call it.  It shares nothing with the HIP path.
 *
 * It is the plain definition of what the step computes, in the paper's order:
 *   Sec. 3.3 ("Potentials of Activation Cache"): the checkpoint is the input
 *       tensor of the decoder layer, so the layer's own pre-attention
 *       LayerNorm is applied to it first (OPT-style pre-LN decoder; the paper
 *       does not print the LayerNorm, this is the reading taken here);
 *   Eq. 7:  [K_c V_c] = A_c x [W_K W_V]          (plus the K and V biases);
 *   Eq. 3:  the regenerated rows are concatenated with the cached rows;
 *   Eq. 4:  AttVal = softmax(Q K^T) V for the one decode query per sequence,
 *           with the usual head_dim^-1/2 score scale (the equation omits it).
 * No tiling, no online softmax, no split over tokens, no fusion: every
 * function is one loop nest a reader can check against the equation.
 *
 * Parallelism: OpenMP over independent rows / (sequence, head) pairs only.
 *
 * Pins (tests/test_oracle_pins.py): LayerNorm, projection and attention are
 * each pinned against closed forms, invariants, brute force in Python loops
 * and torch's CPU library routines; the whole step is pinned by the
 * hand-worked two-token case under tests/golden/ and by ratio and token-order
 * invariance.  No function here is "parity unpinned".
 *
 * Layouts (row-major, last index fastest):
 *   act   [B, L_act, d]     activation checkpoints A_c
 *   gamma, beta [d]         LayerNorm weight / bias
 *   Wkv   [2d, d]           row n holds the input weights of output feature n;
 *                           rows 0..d-1 are the columns of W_K, d..2d-1 of W_V
 *   bkv   [2d]              K bias then V bias
 *   K, V  [B, H, L, dh]     head-major; feature n of a token belongs to head
 *                           n / dh, lane n % dh
 *   q, out [B, H, dh]
 */

#ifndef REAL
#error "include from hybridkv_oracle.c with REAL and SUFFIX defined"
#endif

#define HKO_CAT_(a, b) a##b
#define HKO_CAT(a, b) HKO_CAT_(a, b)
#define HKO(name) HKO_CAT(name, SUFFIX)

/* LayerNorm of M rows of length d: biased variance, two passes, eps inside the
 * square root.  xhat[r, j] = (x[r, j] - mean_r) / sqrt(var_r + eps) * gamma[j] + beta[j]. */
void HKO(hko_layernorm)(const REAL *x, const REAL *gamma, const REAL *beta,
                        int64_t M, int64_t d, REAL eps, REAL *xhat)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < M; ++r) {
        const REAL *xr = x + r * d;
        REAL *yr = xhat + r * d;
        REAL sum = 0;
        for (int64_t j = 0; j < d; ++j) sum += xr[j];
        const REAL mean = sum / (REAL)d;
        REAL sq = 0;
        for (int64_t j = 0; j < d; ++j) {
            const REAL c = xr[j] - mean;
            sq += c * c;
        }
        const REAL var = sq / (REAL)d;
        const REAL rstd = (REAL)1 / HKO_SQRT(var + eps);
        for (int64_t j = 0; j < d; ++j)
            yr[j] = (xr[j] - mean) * rstd * gamma[j] + beta[j];
    }
}

/* Eq. 7 with biases: KV[r, n] = sum_j xhat[r, j] * Wkv[n, j] + bkv[n], n in [0, N).
 * With the full weight (N = 2d) columns 0..d-1 of a row are that token's key and
 * d..2d-1 its value; a caller may pass any subset of the weight rows (and the
 * matching biases) to get only those output features. */
void HKO(hko_kv_projection)(const REAL *xhat, const REAL *Wkv, const REAL *bkv,
                            int64_t M, int64_t d, int64_t N, REAL *KV)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < M; ++r) {
        const REAL *xr = xhat + r * d;
        for (int64_t n = 0; n < N; ++n) {
            const REAL *wn = Wkv + n * d;
            REAL acc = 0;
            for (int64_t j = 0; j < d; ++j) acc += xr[j] * wn[j];
            KV[r * N + n] = acc + bkv[n];
        }
    }
}

/* "KV Gen" (Sec. 4.2.2): LayerNorm -> Eq. 7 -> split features into heads.
 * Writes token t of sequence b to K[b, h, tok_off + t, :] (and V likewise) in
 * tensors whose token axis has length L_cap.  scratch_xhat [B*L_act, d] and
 * scratch_kv [B*L_act, 2d] are caller-provided work arrays. */
void HKO(hko_regen_kv)(const REAL *act, const REAL *gamma, const REAL *beta,
                       const REAL *Wkv, const REAL *bkv,
                       int64_t B, int64_t L_act, int64_t d, int64_t n_heads, REAL eps,
                       REAL *K, REAL *V, int64_t L_cap, int64_t tok_off,
                       REAL *scratch_xhat, REAL *scratch_kv)
{
    const int64_t M = B * L_act;
    const int64_t dh = d / n_heads;
    HKO(hko_layernorm)(act, gamma, beta, M, d, eps, scratch_xhat);
    HKO(hko_kv_projection)(scratch_xhat, Wkv, bkv, M, d, 2 * d, scratch_kv);
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < M; ++r) {
        const int64_t b = r / L_act, t = r % L_act;
        for (int64_t n = 0; n < d; ++n) {
            const int64_t h = n / dh, i = n % dh;
            const int64_t dst = ((b * n_heads + h) * L_cap + tok_off + t) * dh + i;
            K[dst] = scratch_kv[r * 2 * d + n];
            V[dst] = scratch_kv[r * 2 * d + d + n];
        }
    }
}

/* Eq. 4 for one query per (sequence, head): scores over all L tokens, softmax
 * with the maximum subtracted, weighted sum of the value rows.  probs
 * [B, H, L] may be NULL; when given it receives the softmax row. */
void HKO(hko_decode_attention)(const REAL *q, const REAL *K, const REAL *V,
                               int64_t B, int64_t n_heads, int64_t L, int64_t dh,
                               REAL scale, REAL *out, REAL *probs)
{
    const int64_t BH = B * n_heads;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t bh = 0; bh < BH; ++bh) {
        const REAL *qv = q + bh * dh;
        const REAL *Kb = K + bh * L * dh;
        const REAL *Vb = V + bh * L * dh;
        REAL *o = out + bh * dh;
        REAL *p = (REAL *)malloc((size_t)(L > 0 ? L : 1) * sizeof(REAL));
        REAL m = -HKO_INF;
        for (int64_t t = 0; t < L; ++t) {
            REAL s = 0;
            for (int64_t i = 0; i < dh; ++i) s += qv[i] * Kb[t * dh + i];
            s *= scale;
            p[t] = s;
            if (s > m) m = s;
        }
        REAL Z = 0;
        for (int64_t t = 0; t < L; ++t) {
            p[t] = HKO_EXP(p[t] - m);
            Z += p[t];
        }
        for (int64_t i = 0; i < dh; ++i) o[i] = 0;
        for (int64_t t = 0; t < L; ++t) {
            const REAL w = p[t] / Z;
            if (probs) probs[bh * L + t] = w;
            for (int64_t i = 0; i < dh; ++i) o[i] += w * Vb[t * dh + i];
        }
        free(p);
    }
}

/* The whole step.  Context token order is: the L_kv cached tokens, then the
 * L_act regenerated ones (softmax attention does not depend on the order, so
 * which tokens are held in which store is immaterial).  K_full / V_full
 * [B, H, L_kv + L_act, dh] are caller-provided and return the concatenated
 * keys and values (Eq. 3); their regenerated tail is the elementwise
 * comparison target for the GPU's regenerated K/V. */
void HKO(hko_hybrid_decode_attn)(const REAL *q,
                                 const REAL *K_cache, const REAL *V_cache, int64_t L_kv,
                                 const REAL *act, int64_t L_act,
                                 const REAL *gamma, const REAL *beta,
                                 const REAL *Wkv, const REAL *bkv,
                                 int64_t B, int64_t d, int64_t n_heads,
                                 REAL eps, REAL scale,
                                 REAL *out, REAL *K_full, REAL *V_full,
                                 REAL *scratch_xhat, REAL *scratch_kv)
{
    const int64_t dh = d / n_heads;
    const int64_t L = L_kv + L_act;
    /* Eq. 3: cached rows first ... */
    for (int64_t bh = 0; bh < B * n_heads; ++bh)
        for (int64_t t = 0; t < L_kv; ++t)
            for (int64_t i = 0; i < dh; ++i) {
                K_full[(bh * L + t) * dh + i] = K_cache[(bh * L_kv + t) * dh + i];
                V_full[(bh * L + t) * dh + i] = V_cache[(bh * L_kv + t) * dh + i];
            }
    /* ... then the rows regenerated from the checkpoints (Eq. 7). */
    if (L_act > 0)
        HKO(hko_regen_kv)(act, gamma, beta, Wkv, bkv, B, L_act, d, n_heads, eps,
                          K_full, V_full, L, L_kv, scratch_xhat, scratch_kv);
    HKO(hko_decode_attention)(q, K_full, V_full, B, n_heads, L, dh, scale, out, NULL);
}

#undef HKO
#undef HKO_CAT
#undef HKO_CAT_
