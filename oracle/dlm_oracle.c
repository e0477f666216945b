/*
 * CPU fp64 oracle for the dLLM rollout denoising step.  TEST INFRASTRUCTURE ONLY:
 * it exists to check the HIP path and to be timed beside it; no product code
 * path may call it.  It shares no code with the HIP library.
 *
 * Everything here is the plain definition written out, in double precision, on
 * the same bf16 bit patterns the GPU reads (promoted exactly to double).  There
 * is no tiling, no online softmax, no fusion: scores and logits are materialised
 * per row, then reduced.
 *
 *   oracle_attention_rows  softmax(scale * q K^T) V over the keys a query may see.
 *                          The mask predictor of a masked diffusion LM conditions
 *                          on the whole partially masked sequence (Eq. 2), so a
 *                          query sees every key ("full"); a block diffusion LM
 *                          conditions block b on itself and on earlier blocks
 *                          (Eq. 3 and the block partition stated before it), so a
 *                          key is visible iff its block index is <= the query's.
 *   oracle_lmhead_rows     the mask predictor's categorical over the vocabulary
 *                          (Eq. 2) for one position: logits, arg-max token, its
 *                          softmax probability (the "confidence"), log-sum-exp,
 *                          and the runner-up logit.
 *
 * Parity pins: brute force in pure Python on tiny inputs, closed forms and
 * metamorphic identities (tests/test_oracle_*.py).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double bf16_bits_to_double(uint16_t u) {
    uint32_t w = (uint32_t)u << 16;
    float f;
    memcpy(&f, &w, sizeof f);
    return (double)f;
}

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * Attention for a list of (b, h, i) query rows.
 *   q        bf16 bits, element strides q_sb (batch), q_st (query row), q_sh (head); d contiguous
 *   k, v     bf16 bits, the *concatenated* visible context [B, Hkv, Lk, d] with element strides
 *            kv_sb, kv_sh, kv_st; d contiguous
 *   key_pos  [Lk] absolute position of every key (used by the block-causal rule only)
 *   key_ok   optional [B, Lk] bytes; 0 = key absent for that sequence (ragged prefix)
 *   mode     0 full, 1 block-causal with block size bs: key j visible to query i iff
 *            floor(key_pos[j] / bs) <= floor((q_pos0 + i) / bs)
 *   key_rule optional [Lk] (mode 1 only), per key: 0 the rule above; 1 only keys of EARLIER blocks
 *            (block index <); 2 only keys of the query's OWN block (block index ==).  Rules 1 and 2 are
 *            the two halves of block-diffusion training (Eq. 3): the noisy block b is predicted from
 *            itself (rule 2 on the noisy keys) and from the clean blocks before it (rule 1 on the clean keys).
 *   rows     [n, 3] int32 (b, h, i);   GQA: kv head = h / (Hq / Hkv)
 *   out      [n, d] doubles; lse [n] doubles (natural log).  A row that sees no key
 *            gets out = 0 and lse = -inf.
 */
int oracle_attention_rows(const uint16_t *q, int64_t q_sb, int64_t q_st, int64_t q_sh,
                          const uint16_t *k, const uint16_t *v,
                          int64_t kv_sb, int64_t kv_sh, int64_t kv_st,
                          const int32_t *key_pos, const uint8_t *key_ok, const int32_t *key_rule,
                          int32_t Hq, int32_t Hkv, int32_t d, int32_t Lk,
                          int32_t mode, int32_t bs, int32_t q_pos0, double scale,
                          const int32_t *rows, int64_t n_rows,
                          double *out, double *lse) {
    if (Hkv <= 0 || Hq % Hkv != 0 || d <= 0 || Lk < 0) return -1;
    if (mode == 1 && bs <= 0) return -1;
    const int32_t g = Hq / Hkv;
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t r = 0; r < n_rows; ++r) {
        const int32_t b = rows[3 * r + 0], h = rows[3 * r + 1], i = rows[3 * r + 2];
        const int32_t kvh = h / g;
        double *s = (double *)malloc(sizeof(double) * (size_t)(Lk > 0 ? Lk : 1));
        uint8_t *vis = (uint8_t *)malloc((size_t)(Lk > 0 ? Lk : 1));
        if (!s || !vis) { fail = 1; free(s); free(vis); continue; }
        const uint16_t *qrow = q + b * q_sb + i * q_st + h * q_sh;
        double m = -INFINITY;
        for (int32_t j = 0; j < Lk; ++j) {
            int ok = 1;
            if (key_ok && !key_ok[(int64_t)b * Lk + j]) ok = 0;
            if (ok && mode == 1) {
                /* positions are non-negative, so integer division is the floor */
                const int32_t kb = key_pos[j] / bs, qb = (q_pos0 + i) / bs;
                const int32_t rule = key_rule ? key_rule[j] : 0;
                if (rule == 0 && kb > qb) ok = 0;
                if (rule == 1 && kb >= qb) ok = 0;
                if (rule == 2 && kb != qb) ok = 0;
            }
            vis[j] = (uint8_t)ok;
            if (!ok) continue;
            const uint16_t *krow = k + b * kv_sb + kvh * kv_sh + j * kv_st;
            double dot = 0.0;
            for (int32_t c = 0; c < d; ++c)
                dot += bf16_bits_to_double(qrow[c]) * bf16_bits_to_double(krow[c]);
            s[j] = scale * dot;
            if (s[j] > m) m = s[j];
        }
        double *o = out + r * d;
        for (int32_t c = 0; c < d; ++c) o[c] = 0.0;
        if (m == -INFINITY) {            /* no visible key */
            lse[r] = -INFINITY;
            free(s); free(vis);
            continue;
        }
        double l = 0.0;
        for (int32_t j = 0; j < Lk; ++j) {
            if (!vis[j]) continue;
            s[j] = exp(s[j] - m);        /* s now holds p_j */
            l += s[j];
        }
        for (int32_t j = 0; j < Lk; ++j) {
            if (!vis[j]) continue;
            const uint16_t *vrow = v + b * kv_sb + kvh * kv_sh + j * kv_st;
            for (int32_t c = 0; c < d; ++c) o[c] += s[j] * bf16_bits_to_double(vrow[c]);
        }
        for (int32_t c = 0; c < d; ++c) o[c] /= l;
        lse[r] = m + log(l);
        free(s); free(vis);
    }
    return fail ? -2 : 0;
}

/*
 * LM head for M rows.  Row r reads hidden[(row_idx ? row_idx[r] : r) * h_stride + 0..Dh).
 *   z_v   = (sum_k hidden[r,k] * w[v,k]) * inv_T         for v in [0, V)
 *   z_forbid = -inf when forbid >= 0
 *   zmax  = max_v z_v;  tok = smallest v attaining it
 *   lse   = zmax + log sum_v exp(z_v - zmax);  conf = exp(zmax - lse)
 *   z2nd  = max over v != tok of z_v  (-inf when V == 1)
 *   zt[r] = z at target[r] (only when target != NULL): the numerator of log p(target)
 *   nent[r] = sum_v p_v log p_v with p = softmax(z) (optional): the negative entropy of the categorical,
 *             an alternative confidence score (0 for a one-hot distribution, -log V for a uniform one)
 */
int oracle_lmhead_rows(const uint16_t *hidden, int64_t h_stride, const int32_t *row_idx, int64_t M,
                       const uint16_t *w, int64_t w_stride, int32_t Dh, int32_t V,
                       double inv_T, int32_t forbid, const int32_t *target,
                       double *conf, int32_t *tok, double *lse, double *zmax, double *z2nd,
                       double *zt, double *nent) {
    if (V <= 0 || Dh <= 0) return -1;
    double *z = (double *)malloc(sizeof(double) * (size_t)V);
    double *hrow = (double *)malloc(sizeof(double) * (size_t)Dh);
    if (!z || !hrow) { free(z); free(hrow); return -2; }
    for (int64_t r = 0; r < M; ++r) {
        const int64_t src = row_idx ? row_idx[r] : r;
        for (int32_t c = 0; c < Dh; ++c) hrow[c] = bf16_bits_to_double(hidden[src * h_stride + c]);
#pragma omp parallel for schedule(static)
        for (int32_t vv = 0; vv < V; ++vv) {
            const uint16_t *wrow = w + (int64_t)vv * w_stride;
            double dot = 0.0;
            for (int32_t c = 0; c < Dh; ++c) dot += hrow[c] * bf16_bits_to_double(wrow[c]);
            z[vv] = dot * inv_T;
        }
        if (forbid >= 0 && forbid < V) z[forbid] = -INFINITY;
        double m = -INFINITY;
        int32_t arg = 0;
        for (int32_t vv = 0; vv < V; ++vv)
            if (z[vv] > m) { m = z[vv]; arg = vv; }       /* strict >: lowest index wins ties */
        double sum = 0.0, second = -INFINITY;
        for (int32_t vv = 0; vv < V; ++vv) {
            sum += exp(z[vv] - m);
            if (vv != arg && z[vv] > second) second = z[vv];
        }
        const double L = m + log(sum);
        conf[r] = exp(m - L);
        tok[r] = arg;
        lse[r] = L;
        zmax[r] = m;
        z2nd[r] = second;
        if (target && zt) zt[r] = z[target[r]];
        if (nent) {
            double acc = 0.0;
            for (int32_t vv = 0; vv < V; ++vv)
                if (z[vv] > -INFINITY) acc += exp(z[vv] - L) * (z[vv] - L);     /* p log p; p = 0 contributes 0 */
            nent[r] = acc;
        }
    }
    free(z); free(hrow);
    return 0;
}
