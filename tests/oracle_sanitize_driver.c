/* Drives the C oracle over small ragged cases under AddressSanitizer + UndefinedBehaviorSanitizer (host only).
 * Buffers are exactly as large as the documented extents, so any read or write past them is reported.
 * Prints a few values for the Python side to compare with the ordinary build. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_attention_rows(const uint16_t *q, int64_t q_sb, int64_t q_st, int64_t q_sh, const uint16_t *k, const uint16_t *v,
                          int64_t kv_sb, int64_t kv_sh, int64_t kv_st, const int32_t *key_pos, const uint8_t *key_ok,
                          const int32_t *key_rule, int32_t Hq, int32_t Hkv, int32_t d, int32_t Lk, int32_t mode, int32_t bs,
                          int32_t q_pos0, double scale, const int32_t *rows, int64_t n_rows, double *out, double *lse);
int oracle_lmhead_rows(const uint16_t *hidden, int64_t h_stride, const int32_t *row_idx, int64_t M, const uint16_t *w,
                       int64_t w_stride, int32_t Dh, int32_t V, double inv_T, int32_t forbid, const int32_t *target,
                       double *conf, int32_t *tok, double *lse, double *zmax, double *z2nd, double *zt, double *nent);

static uint32_t state = 12345u;
static uint16_t rnd_bf16(void) {            /* a small normal-ish value as bf16 bits */
    float f = 0.f;
    for (int i = 0; i < 4; ++i) {
        state = state * 1664525u + 1013904223u;
        f += (float)(state >> 8) / 16777216.0f - 0.5f;
    }
    uint32_t u;
    memcpy(&u, &f, 4);
    return (uint16_t)(u >> 16);
}
static uint16_t *fill(size_t n) {
    uint16_t *p = (uint16_t *)malloc(n * sizeof(uint16_t));
    for (size_t i = 0; i < n; ++i) p[i] = rnd_bf16();
    return p;
}

int main(void) {
    /* attention: B = 2, Lq = 5, Hq = 6, Hkv = 2, d = 24, Lk = 37; ragged prefix, block-causal with segment rules */
    enum { B = 2, Lq = 5, Hq = 6, Hkv = 2, D = 24, Lk = 37 };
    uint16_t *q = fill((size_t)B * Lq * Hq * D), *k = fill((size_t)B * Hkv * Lk * D), *v = fill((size_t)B * Hkv * Lk * D);
    int32_t key_pos[Lk], key_rule[Lk];
    uint8_t key_ok[B * Lk];
    for (int j = 0; j < Lk; ++j) { key_pos[j] = j; key_rule[j] = j < 12 ? 1 : (j < 30 ? 0 : 2); }
    for (int i = 0; i < B * Lk; ++i) key_ok[i] = (uint8_t)(i % 7 != 3);
    int32_t rows[B * Hq * Lq * 3];
    int n = 0;
    for (int b = 0; b < B; ++b) for (int h = 0; h < Hq; ++h) for (int i = 0; i < Lq; ++i) { rows[3 * n] = b; rows[3 * n + 1] = h; rows[3 * n + 2] = i; ++n; }
    double *out = (double *)malloc(sizeof(double) * n * D), *lse = (double *)malloc(sizeof(double) * n);
    for (int mode = 0; mode < 2; ++mode) {
        int rc = oracle_attention_rows(q, (int64_t)Lq * Hq * D, (int64_t)Hq * D, D, k, v, (int64_t)Hkv * Lk * D, (int64_t)Lk * D, D,
                                       key_pos, key_ok, mode ? key_rule : NULL, Hq, Hkv, D, Lk, mode, 4, 9, 1.0 / sqrt((double)D),
                                       rows, n, out, lse);
        if (rc) { printf("attention rc %d\n", rc); return 1; }
        double s = 0; for (int i = 0; i < n * D; ++i) s += out[i];
        printf("attn mode %d sum %.12f lse0 %.12f\n", mode, s, lse[0]);
    }
    /* a query that sees nothing: every key absent */
    memset(key_ok, 0, sizeof key_ok);
    if (oracle_attention_rows(q, (int64_t)Lq * Hq * D, (int64_t)Hq * D, D, k, v, (int64_t)Hkv * Lk * D, (int64_t)Lk * D, D, key_pos, key_ok, NULL,
                              Hq, Hkv, D, Lk, 0, 0, 0, 0.2, rows, 3, out, lse)) return 1;
    printf("attn empty out0 %.3f lse0 %s\n", out[0], isinf(lse[0]) && lse[0] < 0 ? "-inf" : "finite");
    /* zero keys at all */
    if (oracle_attention_rows(q, (int64_t)Lq * Hq * D, (int64_t)Hq * D, D, k, v, 0, 0, D, key_pos, NULL, NULL, Hq, Hkv, D, 0, 0, 0, 0, 0.2, rows, 2, out, lse)) return 1;
    /* LM head: gathered rows, ragged V, forbidden token, target and entropy outputs; then V = 1 */
    enum { R = 9, M = 4, Dh = 40, V = 77 };
    uint16_t *hid = fill((size_t)R * Dh), *w = fill((size_t)V * Dh);
    int32_t row_idx[M] = {8, 0, 3, 8}, target[M] = {0, 76, 5, 40}, tok[M];
    double conf[M], l2[M], zmax[M], z2nd[M], zt[M], nent[M];
    if (oracle_lmhead_rows(hid, Dh, row_idx, M, w, Dh, Dh, V, 0.7, V - 1, target, conf, tok, l2, zmax, z2nd, zt, nent)) return 1;
    printf("lm conf %.12f %.12f tok %d %d nent %.12f\n", conf[0], conf[3], tok[0], tok[2], nent[1]);
    if (oracle_lmhead_rows(hid, Dh, NULL, M, w, Dh, Dh, V, 1.0, -1, NULL, conf, tok, l2, zmax, z2nd, NULL, NULL)) return 1;
    if (oracle_lmhead_rows(hid, Dh, NULL, 2, w, Dh, Dh, 1, 1.0, -1, NULL, conf, tok, l2, zmax, z2nd, NULL, NULL)) return 1;
    printf("lm V=1 conf %.3f tok %d z2nd %s\n", conf[0], tok[0], isinf(z2nd[0]) ? "-inf" : "finite");
    if (oracle_lmhead_rows(hid, Dh, NULL, 0, w, Dh, Dh, V, 1.0, -1, NULL, conf, tok, l2, zmax, z2nd, NULL, NULL)) return 1;
    free(q); free(k); free(v); free(out); free(lse); free(hid); free(w);
    printf("ok\n");
    return 0;
}
