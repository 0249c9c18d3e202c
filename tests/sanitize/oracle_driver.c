/* Runs every entry point of the CPU oracle on small, ragged inputs in exactly-sized heap buffers, for a build with
 * -fsanitize=address,undefined: an access outside a buffer, a misaligned or overflowing operation aborts the run.
 * The numbers are checked elsewhere (tests/test_oracle_pins.py); this program only has to finish and print "ok". */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

double ora_decode_e4m3(uint8_t code);
double ora_decode_bf16(uint16_t bits);
double ora_decode_e8m0(uint8_t code);
double ora_decode_e2m1(uint8_t code);
int ora_decode_mx(const uint8_t *elems, const uint8_t *scales, double *dst, size_t rows, int d, int kind);
int ora_bidir_attention(const void *Q, const void *K, const void *V, double *O, int B, int H, int Hkv, int N, int d,
                        int qk_dtype, int v_dtype, const float *q_scale, const float *k_scale, const int32_t *rows, int nrows);
int ora_block_attention_cached(const void *Qblk, const void *Kc, const void *Vc, double *O, int block_start, int block_len,
                               const void *Kblk, const void *Vblk, int B, int H, int Hkv, int N, int d, int qk_dtype,
                               int v_dtype, const float *q_scale, const float *k_scale, const int32_t *rows, int nrows);
int ora_verify_scores(const void *logits_d, const void *logits_v, int P, int V, int dtype, const int32_t *rows, int nrows,
                      double *kl, double *conf, int32_t *tok);
void ora_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);
double ora_row_uniform(uint64_t seed, uint64_t row);
int ora_remask_decide(const float *score32, const uint8_t *mask, int mode, float threshold, uint64_t seed, int B, int G,
                      uint8_t *out_mask, double *prob);
int ora_unmask_decide(const float *conf32, const uint8_t *mask, int mode, float threshold, int B, int G, uint8_t *out_mask);

static uint32_t lcg = 12345u;
static uint32_t rnd(void) { lcg = lcg * 1664525u + 1013904223u; return lcg >> 8; }
static float rndf(void) { return (float)((int)(rnd() % 2001) - 1000) / 500.0f; }

static void *fill(size_t n, int dtype)   /* n elements of storage type dtype (0 f32, 1 bf16, 2 e4m3), exact size */
{
    size_t eb = dtype == 0 ? 4 : dtype == 1 ? 2 : 1;
    unsigned char *p = malloc(n * eb > 0 ? n * eb : 1);
    for (size_t i = 0; i < n; ++i) {
        float f = rndf();
        if (dtype == 0) memcpy(p + 4 * i, &f, 4);
        else if (dtype == 1) { uint32_t u; memcpy(&u, &f, 4); uint16_t h = (uint16_t)(u >> 16); memcpy(p + 2 * i, &h, 2); }
        else { uint8_t c = (uint8_t)(rnd() & 0xFF); if ((c & 0x7F) == 0x7F) c = 0x3A; p[i] = c; }
    }
    return p;
}

static int attention_case(int B, int H, int Hkv, int N, int d, int qk, int v, int bl, int bs)
{
    void *Q = fill((size_t)B * H * N * d, qk), *K = fill((size_t)B * Hkv * N * d, qk), *V = fill((size_t)B * Hkv * N * d, v);
    float *qs = malloc(sizeof(float) * B * H), *ks = malloc(sizeof(float) * B * Hkv);
    for (int i = 0; i < B * H; ++i) qs[i] = 0.5f + 0.01f * i;
    for (int i = 0; i < B * Hkv; ++i) ks[i] = 0.7f + 0.02f * i;
    double *O = malloc(sizeof(double) * (size_t)B * H * N * d);
    int rc = ora_bidir_attention(Q, K, V, O, B, H, Hkv, N, d, qk, v, qs, ks, NULL, 0);
    int32_t rows[6] = {0, 0, 0, B - 1, H - 1, N - 1};
    double *Or = malloc(sizeof(double) * 2 * d);
    rc |= ora_bidir_attention(Q, K, V, Or, B, H, Hkv, N, d, qk, v, NULL, NULL, rows, 2);
    void *Qb = fill((size_t)B * H * bl * d, qk), *Kb = fill((size_t)B * Hkv * bl * d, qk), *Vb = fill((size_t)B * Hkv * bl * d, v);
    double *Ob = malloc(sizeof(double) * (size_t)B * H * bl * d);
    rc |= ora_block_attention_cached(Qb, K, V, Ob, bs, bl, Kb, Vb, B, H, Hkv, N, d, qk, v, qs, ks, NULL, 0);
    rc |= ora_block_attention_cached(Qb, K, V, Ob, bs, bl, NULL, NULL, B, H, Hkv, N, d, qk, v, NULL, NULL, NULL, 0);
    int32_t brow[3] = {B - 1, H - 1, bl - 1};
    rc |= ora_block_attention_cached(Qb, K, V, Or, bs, bl, Kb, Vb, B, H, Hkv, N, d, qk, v, qs, ks, brow, 1);
    for (size_t i = 0; i < (size_t)B * H * N * d; ++i) if (!isfinite(O[i])) rc |= 2;
    /* arguments the oracle must refuse without touching anything */
    if (ora_block_attention_cached(Qb, K, V, Ob, N - bl + 1, bl, Kb, Vb, B, H, Hkv, N, d, qk, v, qs, ks, NULL, 0) == 0) rc |= 4;
    int32_t bad[3] = {B, 0, 0};
    if (ora_bidir_attention(Q, K, V, Or, B, H, Hkv, N, d, qk, v, NULL, NULL, bad, 1) == 0) rc |= 8;
    free(Q); free(K); free(V); free(qs); free(ks); free(O); free(Or); free(Qb); free(Kb); free(Vb); free(Ob);
    return rc;
}

static int verify_case(int B, int G, int V, int dtype)
{
    int P = B * G, rc = 0;
    void *ld = fill((size_t)P * V, dtype), *lv = fill((size_t)P * V, dtype);
    double *kl = malloc(sizeof(double) * P), *conf = malloc(sizeof(double) * P), *prob = malloc(sizeof(double) * P);
    int32_t *tok = malloc(sizeof(int32_t) * P);
    rc |= ora_verify_scores(ld, lv, P, V, dtype, NULL, P, kl, conf, tok);
    rc |= ora_verify_scores(NULL, lv, P, V, dtype, NULL, P, kl, conf, tok);
    int32_t rows[2] = {P - 1, 0};
    double kl2[2], conf2[2];
    int32_t tok2[2];
    rc |= ora_verify_scores(ld, lv, P, V, dtype, rows, 2, kl2, conf2, tok2);
    rc |= ora_verify_scores(ld, lv, P, V, dtype, NULL, P, kl, conf, tok);
    float *s32 = malloc(sizeof(float) * P);
    uint8_t *mask = malloc(P), *om = malloc(P);
    for (int i = 0; i < P; ++i) { s32[i] = (float)kl[i]; mask[i] = (uint8_t)(rnd() % 3 == 0); }
    for (int mode = 0; mode <= 6; ++mode)
        rc |= ora_remask_decide(s32, mask, mode, mode >= 5 ? 3.0f : 0.3f, 77u + mode, B, G, om, prob);
    for (int i = 0; i < P; ++i) s32[i] = (float)conf[i];
    for (int mode = 0; mode <= 1; ++mode)
        rc |= ora_unmask_decide(s32, mask, mode, mode ? 2.0f : 0.01f, B, G, om);
    if (ora_remask_decide(s32, mask, 9, 0.f, 0, B, G, om, prob) == 0) rc |= 16;
    free(ld); free(lv); free(kl); free(conf); free(prob); free(tok); free(s32); free(mask); free(om);
    return rc;
}

int main(void)
{
    int rc = 0;
    for (int c = 0; c < 256; ++c) (void)ora_decode_e4m3((uint8_t)c);
    for (int b = 0; b < 65536; b += 257) (void)ora_decode_bf16((uint16_t)b);
    uint32_t ctr[4] = {1, 2, 3, 4}, key[2] = {5, 6}, out[4];
    ora_philox4x32_10(ctr, key, out);
    (void)ora_row_uniform(0xFFFFFFFFFFFFFFFFull, 0xFFFFFFFFFFFFFFFFull);
    rc |= attention_case(1, 2, 2, 1, 64, 1, 1, 1, 0);
    rc |= attention_case(2, 4, 2, 37, 64, 1, 1, 5, 32);
    rc |= attention_case(1, 3, 1, 50, 128, 2, 1, 16, 17);
    rc |= attention_case(2, 2, 1, 33, 64, 0, 0, 7, 0);
    for (int c = 0; c < 256; ++c) { (void)ora_decode_e8m0((uint8_t)c); (void)ora_decode_e2m1((uint8_t)(c & 15)); }
    {
        /* block-scaled tensors, exactly sized: 3 rows of 64 elements (e4m3: 192 bytes, e2m1: 96), 6 scales; decoded
         * values attended as fp64 (dtype 3) */
        enum { R = 3, D = 64 };
        uint8_t *e8 = malloc(R * D), *e4 = malloc(R * D / 2), *sc = malloc(R * D / 32);
        double *dq = malloc(sizeof(double) * R * D), *dv = malloc(sizeof(double) * R * D), *o = malloc(sizeof(double) * R * D);
        for (int i = 0; i < R * D; ++i) e8[i] = (uint8_t)((i * 37) % 0x7E);
        for (int i = 0; i < R * D / 2; ++i) e4[i] = (uint8_t)(i * 29);
        for (int i = 0; i < R * D / 32; ++i) sc[i] = (uint8_t)(120 + i);
        rc |= ora_decode_mx(e8, sc, dq, R, D, 0);
        rc |= ora_decode_mx(e4, sc, dv, R, D, 1);
        if (ora_decode_mx(e8, sc, dq, R, 48, 0) == 0) rc |= 32;          /* d not a multiple of 32 */
        rc |= ora_bidir_attention(dq, dq, dv, o, 1, 1, 1, R, D, 3, 3, NULL, NULL, NULL, 0);
        free(e8); free(e4); free(sc); free(dq); free(dv); free(o);
    }
    rc |= verify_case(1, 1, 8, 1);
    rc |= verify_case(3, 7, 1000, 1);
    rc |= verify_case(2, 5, 37, 0);
    if (rc != 0) { printf("FAILED rc=%d\n", rc); return 1; }
    printf("ok\n");
    return 0;
}
