/*
 * TEST INFRASTRUCTURE -- CPU oracle for one DualDiffusion draft-then-verify step.
 *
 * A plain, slow, fp64 implementation of what the hot path computes, written from
 * the paper's definitions.  Only tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it; the product path never does.  It shares no code,
 * header, table or constant with the HIP library.
 *
 *   attention            softmax(Q K^T / sqrt(d_k)) V, the form of Eq. 3 (Sec. 2.2),
 *                        taken over ALL positions because the verifier's attention
 *                        is bidirectional (Sec. 2.2: no position is hidden from any
 *                        other); Alg. 1's verification line needs it at every
 *                        position.
 *   block attention      the same formula for the active block's queries only, with
 *                        keys/values of the other positions read from a (possibly
 *                        stale) cache -- the block-wise approximate KV cache of
 *                        Sec. 2.3 that the drafter of Sec. 3.1 runs on.
 *   verify scores        per position: verifier confidence c_V = max_x p_V(x) (Eq. 7),
 *                        its argmax, and KL(p_D || p_V) (Eq. 5), natural log.
 *   remask decision      Trust Verifier (Eq. 4: change nothing), KL threshold
 *                        (remask iff KL > tau), KL probabilistic (Eq. 6), confidence
 *                        threshold (remask iff c_V < tau) and confidence
 *                        probabilistic (remask w.p. 1 - c_V), Sec. 3.2.
 *
 * Everything is two-pass and untiled: scores are materialised per query row, the
 * maximum is subtracted, exponentials are summed.  Storage types are decoded
 * exactly into double (fp32 and bf16 are subsets of double; fp8 is OCP e4m3).
 *
 * The paper states no storage precision (Sec. 4.1 runs stock models); the reduced-
 * precision workloads are input formats only.  Block-scaled ("MX") tensors follow
 * the OCP Microscaling Formats specification v1.0: 32 consecutive elements along
 * the head dimension share one power-of-two scale (E8M0); they are decoded to
 * double by ora_decode_mx and then go through the same attention as any other
 * input (dtype ORA_F64).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORA_F32 = 0, ORA_BF16 = 1, ORA_FP8_E4M3 = 2, ORA_F64 = 3 };
enum { ORA_MX_E4M3 = 0, ORA_MX_E2M1 = 1 };
enum { ORA_TRUST = 0, ORA_KL_THRESH = 1, ORA_CONF_THRESH = 2, ORA_KL_PROB = 3, ORA_CONF_PROB = 4,
       ORA_KL_TOPK = 5, ORA_CONF_TOPK = 6 };

/* ---------------------------------------------------------------- decoding */

/* OCP 8-bit float, 4 exponent bits (bias 7), 3 mantissa bits, no infinities;
 * exponent 15 with mantissa 7 is NaN; exponent 0 is subnormal (m/8 * 2^-6). */
double ora_decode_e4m3(uint8_t code)
{
    int s = code >> 7, e = (code >> 3) & 15, m = code & 7;
    double v;
    if (e == 15 && m == 7)
        v = NAN;
    else if (e == 0)
        v = ldexp((double)m / 8.0, -6);
    else
        v = ldexp(1.0 + (double)m / 8.0, e - 7);
    return s ? -v : v;
}

/* bf16 = the upper half of an IEEE fp32 pattern */
double ora_decode_bf16(uint16_t bits)
{
    uint32_t u = (uint32_t)bits << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* E8M0 scale of a block-scaled format: 8 exponent bits, bias 127, no sign, no mantissa:
 * 2^(code - 127); code 255 is NaN. */
double ora_decode_e8m0(uint8_t code)
{
    if (code == 255)
        return NAN;
    return ldexp(1.0, (int)code - 127);
}

/* 4-bit float: sign, 2 exponent bits (bias 1), 1 mantissa bit; no NaN, no infinity.
 * exponent 0 is subnormal (m/2 * 2^0): the values are +-{0, 0.5, 1, 1.5, 2, 3, 4, 6}. */
double ora_decode_e2m1(uint8_t code)
{
    int s = (code >> 3) & 1, e = (code >> 1) & 3, m = code & 1;
    double v = e == 0 ? (double)m / 2.0 : ldexp(1.0 + (double)m / 2.0, e - 1);
    return s ? -v : v;
}

/* Block-scaled tensor -> double.  `rows` rows of d elements; element c of a row belongs to block c / 32,
 * whose scale is scales[row * (d / 32) + c / 32]; value = element x scale.  kind ORA_MX_E4M3: one byte per
 * element; ORA_MX_E2M1: two elements per byte, the even element in the low four bits.  d % 32 == 0. */
int ora_decode_mx(const uint8_t *elems, const uint8_t *scales, double *dst, size_t rows, int d, int kind)
{
    if (!elems || !scales || !dst || d <= 0 || d % 32 || (kind != ORA_MX_E4M3 && kind != ORA_MX_E2M1))
        return -1;
    for (size_t r = 0; r < rows; ++r)
        for (int c = 0; c < d; ++c) {
            size_t i = r * (size_t)d + (size_t)c;
            double x = kind == ORA_MX_E4M3 ? ora_decode_e4m3(elems[i])
                                           : ora_decode_e2m1((uint8_t)((elems[i / 2] >> (4 * (i & 1))) & 15));
            dst[i] = x * ora_decode_e8m0(scales[r * (size_t)(d / 32) + (size_t)(c / 32)]);
        }
    return 0;
}

static double load_elem(const void *base, size_t idx, int dtype)
{
    switch (dtype) {
    case ORA_F32: return (double)((const float *)base)[idx];
    case ORA_BF16: return ora_decode_bf16(((const uint16_t *)base)[idx]);
    case ORA_F64: return ((const double *)base)[idx];
    default: return ora_decode_e4m3(((const uint8_t *)base)[idx]);
    }
}

/* decode `count` consecutive elements starting at element offset `off`, times `scale` */
static void decode_run(double *dst, const void *base, size_t off, size_t count, int dtype, double scale)
{
    for (size_t i = 0; i < count; ++i)
        dst[i] = scale * load_elem(base, off + i, dtype);
}

/* ---------------------------------------------------------------- attention */

/* One query row against N key/value rows (already decoded to double):
 * s_j = (q . k_j) / sqrt(d);  w_j = exp(s_j - max_j s_j);  o = sum_j w_j v_j / sum_j w_j. */
static void attend_one_row(const double *q, const double *Kd, const double *Vd, int N, int d,
                           double *scores, double *o)
{
    const double inv_sqrt_d = 1.0 / sqrt((double)d);
    double m = -INFINITY;
    for (int j = 0; j < N; ++j) {
        double s = 0.0;
        for (int c = 0; c < d; ++c)
            s += q[c] * Kd[(size_t)j * d + c];
        s *= inv_sqrt_d;
        scores[j] = s;
        if (s > m)
            m = s;
    }
    double denom = 0.0;
    for (int c = 0; c < d; ++c)
        o[c] = 0.0;
    for (int j = 0; j < N; ++j) {
        double w = exp(scores[j] - m);
        denom += w;
        for (int c = 0; c < d; ++c)
            o[c] += w * Vd[(size_t)j * d + c];
    }
    for (int c = 0; c < d; ++c)
        o[c] /= denom;
}

/* Decoded keys and values one query head sees: head h of batch b reads kv head
 * floor(h * Hkv / H); row j comes from the block tensors when they are given and
 * block_start <= j < block_start + block_len, else from the (cache) tensors K, V. */
static void gather_kv(double *Kd, double *Vd, const void *K, const void *V, const void *Kblk, const void *Vblk,
                      int b, int h, int H, int Hkv, int N, int d, int qk_dtype, int v_dtype,
                      const float *k_scale, const float *v_scale, int block_start, int block_len)
{
    int kvh = (int)(((long)h * Hkv) / H);
    double ks = k_scale ? (double)k_scale[(size_t)b * Hkv + kvh] : 1.0;
    double vs = v_scale ? (double)v_scale[(size_t)b * Hkv + kvh] : 1.0;   /* real value = scale x decoded value */
    for (int j = 0; j < N; ++j) {
        int in_block = Kblk && j >= block_start && j < block_start + block_len;
        if (in_block) {
            size_t off = (((size_t)b * Hkv + kvh) * block_len + (size_t)(j - block_start)) * d;
            decode_run(Kd + (size_t)j * d, Kblk, off, d, qk_dtype, ks);
            decode_run(Vd + (size_t)j * d, Vblk, off, d, v_dtype, vs);
        } else {
            size_t off = (((size_t)b * Hkv + kvh) * N + (size_t)j) * d;
            decode_run(Kd + (size_t)j * d, K, off, d, qk_dtype, ks);
            decode_run(Vd + (size_t)j * d, V, off, d, v_dtype, vs);
        }
    }
}

/*
 * General entry: Q is [B,H,Nq,d]; K,V are [B,Hkv,N,d]; optional Kblk,Vblk [B,Hkv,block_len,d].
 * rows == NULL : every (b,h,i) row is computed, O is [B,H,Nq,d] (double).
 * rows != NULL : rows is [nrows][3] = (b,h,i); O is [nrows][d].
 * returns 0, or -1 on a bad argument.
 */
int ora_attention_vs(const void *Q, const void *K, const void *V, double *O,
                     int B, int H, int Hkv, int Nq, int N, int d, int qk_dtype, int v_dtype,
                     const float *q_scale, const float *k_scale, const float *v_scale,
                     const void *Kblk, const void *Vblk, int block_start, int block_len,
                     const int32_t *rows, int nrows);

int ora_attention(const void *Q, const void *K, const void *V, double *O,
                  int B, int H, int Hkv, int Nq, int N, int d, int qk_dtype, int v_dtype,
                  const float *q_scale, const float *k_scale,
                  const void *Kblk, const void *Vblk, int block_start, int block_len,
                  const int32_t *rows, int nrows)
{
    return ora_attention_vs(Q, K, V, O, B, H, Hkv, Nq, N, d, qk_dtype, v_dtype, q_scale, k_scale, NULL,
                            Kblk, Vblk, block_start, block_len, rows, nrows);
}

/* The same with a per-(batch, kv head) multiplier of the decoded values of V as well (v_scale [B*Hkv] or NULL):
 * the second precision workload stores V in e4m3 like K, one fp32 scale per head. */
int ora_attention_vs(const void *Q, const void *K, const void *V, double *O,
                     int B, int H, int Hkv, int Nq, int N, int d, int qk_dtype, int v_dtype,
                     const float *q_scale, const float *k_scale, const float *v_scale,
                     const void *Kblk, const void *Vblk, int block_start, int block_len,
                     const int32_t *rows, int nrows)
{
    if (!Q || !K || !V || !O || B < 0 || H <= 0 || Hkv <= 0 || H % Hkv || Nq < 0 || N <= 0 || d <= 0)
        return -1;
    if ((Kblk == NULL) != (Vblk == NULL))
        return -1;
    if (Kblk && (block_start < 0 || block_len < 0 || block_start + block_len > N))
        return -1;

    if (rows) {
        int bad = 0;
#pragma omp parallel for schedule(dynamic)
        for (int r = 0; r < nrows; ++r) {
            int b = rows[3 * r], h = rows[3 * r + 1], i = rows[3 * r + 2];
            if (b < 0 || b >= B || h < 0 || h >= H || i < 0 || i >= Nq) {
                bad = 1;
                continue;
            }
            double *Kd = malloc(sizeof(double) * (size_t)N * d);
            double *Vd = malloc(sizeof(double) * (size_t)N * d);
            double *sc = malloc(sizeof(double) * (size_t)N);
            double *q = malloc(sizeof(double) * (size_t)d);
            gather_kv(Kd, Vd, K, V, Kblk, Vblk, b, h, H, Hkv, N, d, qk_dtype, v_dtype, k_scale, v_scale, block_start, block_len);
            double qs = q_scale ? (double)q_scale[(size_t)b * H + h] : 1.0;
            decode_run(q, Q, (((size_t)b * H + h) * Nq + (size_t)i) * d, d, qk_dtype, qs);
            attend_one_row(q, Kd, Vd, N, d, sc, O + (size_t)r * d);
            free(Kd); free(Vd); free(sc); free(q);
        }
        return bad ? -1 : 0;
    }

    const int chunk = 32;
    const int nchunks = (Nq + chunk - 1) / chunk;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int bh = 0; bh < B * H; ++bh) {
        for (int ch = 0; ch < nchunks; ++ch) {
            int b = bh / H, h = bh % H;
            double *Kd = malloc(sizeof(double) * (size_t)N * d);
            double *Vd = malloc(sizeof(double) * (size_t)N * d);
            double *sc = malloc(sizeof(double) * (size_t)N);
            double *q = malloc(sizeof(double) * (size_t)d);
            gather_kv(Kd, Vd, K, V, Kblk, Vblk, b, h, H, Hkv, N, d, qk_dtype, v_dtype, k_scale, v_scale, block_start, block_len);
            double qs = q_scale ? (double)q_scale[(size_t)b * H + h] : 1.0;
            int i1 = (ch + 1) * chunk < Nq ? (ch + 1) * chunk : Nq;
            for (int i = ch * chunk; i < i1; ++i) {
                size_t row = ((size_t)b * H + h) * Nq + (size_t)i;
                decode_run(q, Q, row * d, d, qk_dtype, qs);
                attend_one_row(q, Kd, Vd, N, d, sc, O + row * d);
            }
            free(Kd); free(Vd); free(sc); free(q);
        }
    }
    return 0;
}

/* Verifier attention: every position attends every position (Sec. 2.2). */
int ora_bidir_attention(const void *Q, const void *K, const void *V, double *O,
                        int B, int H, int Hkv, int N, int d, int qk_dtype, int v_dtype,
                        const float *q_scale, const float *k_scale, const int32_t *rows, int nrows)
{
    return ora_attention(Q, K, V, O, B, H, Hkv, N, N, d, qk_dtype, v_dtype, q_scale, k_scale,
                         NULL, NULL, 0, 0, rows, nrows);
}

/* Drafter attention: only the block's queries; other positions come from the cache (Sec. 2.3). */
int ora_block_attention_cached(const void *Qblk, const void *Kc, const void *Vc, double *O,
                               int block_start, int block_len, const void *Kblk, const void *Vblk,
                               int B, int H, int Hkv, int N, int d, int qk_dtype, int v_dtype,
                               const float *q_scale, const float *k_scale, const int32_t *rows, int nrows)
{
    if (block_start < 0 || block_len <= 0 || block_start + block_len > N)
        return -1;
    return ora_attention(Qblk, Kc, Vc, O, B, H, Hkv, block_len, N, d, qk_dtype, v_dtype, q_scale, k_scale,
                         Kblk, Vblk, block_start, block_len, rows, nrows);
}

/* ---------------------------------------------------------------- verification scores */

/* log-softmax of one row into logp[0..V); returns the index of the first maximum. */
static int row_log_softmax(const void *logits, size_t off, int V, int dtype, double *logp)
{
    double m = -INFINITY;
    int arg = 0;
    for (int x = 0; x < V; ++x) {
        double l = load_elem(logits, off + x, dtype);
        logp[x] = l;
        if (l > m) {
            m = l;
            arg = x;
        }
    }
    double z = 0.0;
    for (int x = 0; x < V; ++x)
        z += exp(logp[x] - m);
    double lse = m + log(z);
    for (int x = 0; x < V; ++x)
        logp[x] -= lse;
    return arg;
}

/*
 * Per-row statistics for the listed rows (rows == NULL: all P rows, in order).
 *   conf[r]  = max_x p_V(x)                       (Eq. 7)
 *   token[r] = lowest index attaining that max
 *   kl[r]    = sum_x p_D(x) (log p_D(x) - log p_V(x))   (Eq. 5); NaN when logits_d == NULL
 * A vocabulary entry with p_D(x) = 0 contributes nothing to the KL sum.
 */
int ora_verify_scores(const void *logits_d, const void *logits_v, int P, int V, int dtype,
                      const int32_t *rows, int nrows, double *kl, double *conf, int32_t *token)
{
    if (!logits_v || P < 0 || V <= 0 || !kl || !conf || !token)
        return -1;
    int n = rows ? nrows : P;
    int bad = 0;
#pragma omp parallel for schedule(dynamic)
    for (int r = 0; r < n; ++r) {
        int i = rows ? rows[r] : r;
        if (i < 0 || i >= P) {
            bad = 1;
            continue;
        }
        double *lpv = malloc(sizeof(double) * (size_t)V);
        int arg = row_log_softmax(logits_v, (size_t)i * V, V, dtype, lpv);
        token[r] = arg;
        conf[r] = exp(lpv[arg]);
        if (logits_d) {
            double *lpd = malloc(sizeof(double) * (size_t)V);
            row_log_softmax(logits_d, (size_t)i * V, V, dtype, lpd);
            double acc = 0.0;
            for (int x = 0; x < V; ++x) {
                double pd = exp(lpd[x]);
                if (pd > 0.0)
                    acc += pd * (lpd[x] - lpv[x]);
            }
            kl[r] = acc;
            free(lpd);
        } else {
            kl[r] = NAN;
        }
        free(lpv);
    }
    return bad ? -1 : 0;
}

/* ---------------------------------------------------------------- counter-based uniforms */

/* Philox-4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw: "Parallel random numbers:
 * as easy as 1, 2, 3", SC'11).  Each round multiplies words 0 and 2 of the counter by
 * two fixed odd constants, keeps high and low halves, and mixes in the key, which is
 * advanced by two Weyl constants between rounds. */
void ora_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The uniform in [0,1) attached to verified row `row` under `seed`:
 * counter = (row low word, row high word, 0, 0), key = (seed low word, seed high word),
 * u = top 24 bits of output word 0, times 2^-24. */
double ora_row_uniform(uint64_t seed, uint64_t row)
{
    uint32_t ctr[4] = { (uint32_t)row, (uint32_t)(row >> 32), 0u, 0u };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t out[4];
    ora_philox4x32_10(ctr, key, out);
    return (double)(out[0] >> 8) * (1.0 / 16777216.0);
}

/* ---------------------------------------------------------------- remask decision */

/*
 * mask[i] = 1: position i still holds [MASK]; 0: decoded, hence eligible for remasking
 * (the KL and confidence rules are stated for unmasked positions, Sec. 3.2.2 / 3.2.3).
 * score32[i] is the per-row score rounded to fp32 (KL in the KL modes, confidence
 * otherwise); the decision is taken on that fp32 value against the fp32 threshold.
 *
 *   TRUST        nothing is remasked (Eq. 4)
 *   KL_THRESH    remask iff KL > tau
 *   CONF_THRESH  remask iff c_V < tau
 *   KL_PROB      remask iff u_i < KL_i / sum_{j eligible, same sequence} KL_j   (Eq. 6);
 *                negative round-off in KL is clamped to 0; an empty or all-zero sum remasks nothing
 *   CONF_PROB    remask iff u_i < 1 - c_V
 *   KL_TOPK      budgeted forms of the two threshold rules (a variant, not a rule of the paper): of each
 *   CONF_TOPK    sequence's eligible positions the k = floor(tau) worst are remasked - largest KL, or
 *                smallest c_V; equal scores: the lower position first.  Written as the definition:
 *                position i is remasked iff fewer than k eligible positions are worse than it.
 *
 * out_mask[i] = mask[i] OR remask_i.  prob[i] (optional) receives the remask probability
 * used in the probabilistic modes (0 elsewhere), so that a test can exempt draws that
 * fall within rounding distance of it.
 */
int ora_remask_decide(const float *score32, const uint8_t *mask, int mode, float threshold, uint64_t seed,
                      int B, int G, uint8_t *out_mask, double *prob)
{
    if (!score32 || !mask || !out_mask || B < 0 || G < 0)
        return -1;
    if (mode < ORA_TRUST || mode > ORA_CONF_TOPK)
        return -1;
    if ((mode == ORA_KL_TOPK || mode == ORA_CONF_TOPK) && !(threshold >= 0.0f && threshold <= 3.0e38f))
        return -1;
    for (int b = 0; b < B; ++b) {
        double total = 0.0;
        if (mode == ORA_KL_PROB)
            for (int g = 0; g < G; ++g) {
                size_t i = (size_t)b * G + g;
                if (mask[i] == 0 && score32[i] > 0.0f)
                    total += (double)score32[i];
            }
        for (int g = 0; g < G; ++g) {
            size_t i = (size_t)b * G + g;
            int eligible = mask[i] == 0;
            int remask = 0;
            double p = 0.0;
            switch (mode) {
            case ORA_TRUST:
                break;
            case ORA_KL_THRESH:
                remask = score32[i] > threshold;
                break;
            case ORA_CONF_THRESH:
                remask = score32[i] < threshold;
                break;
            case ORA_KL_PROB: {
                double k = score32[i] > 0.0f ? (double)score32[i] : 0.0;
                p = total > 0.0 ? k / total : 0.0;
                remask = ora_row_uniform(seed, (uint64_t)i) < p;
                break;
            }
            case ORA_CONF_PROB:
                p = 1.0 - (double)score32[i];
                remask = ora_row_uniform(seed, (uint64_t)i) < p;
                break;
            case ORA_KL_TOPK:
            case ORA_CONF_TOPK: {
                double worse = 0.0;                       /* eligible positions of this sequence worse than g */
                for (int h = 0; h < G; ++h) {
                    size_t j = (size_t)b * G + h;
                    if (mask[j] != 0)
                        continue;
                    int more = mode == ORA_KL_TOPK ? score32[j] > score32[i] : score32[j] < score32[i];
                    if (more || (score32[j] == score32[i] && h < g))
                        worse += 1.0;
                }
                remask = worse < floor((double)threshold);
                break;
            }
            }
            out_mask[i] = (uint8_t)(mask[i] != 0 || (eligible && remask));
            if (prob)
                prob[i] = eligible ? p : 0.0;
        }
    }
    return 0;
}

/* ---------------------------------------------------------------- drafter unmasking step */

/*
 * x <- Unmask(p_D, x) of Alg. 1 (drafting phase): of the positions that still hold [MASK] (mask[i] != 0)
 * a subset is revealed according to the drafter's confidence c_D,i = max_x p_D(x | i) (Sec. 2.1), given here
 * rounded to fp32.  Selection rules (Sec. 2.3 names both):
 *   mode 0  every candidate with c_D,i > tau, and in any case the most confident candidate of the sequence
 *           (so that each step reveals something; the paper leaves the empty case open)
 *   mode 1  a fixed number per step: the k = floor(tau) most confident candidates
 * "more confident" = larger c_D, equal values: the lower position.  Written as the definition: the rank of
 * a candidate is the number of candidates of its sequence that are more confident than it.
 * out_mask[i] = mask[i] != 0 and not selected_i.
 */
int ora_unmask_decide(const float *conf32, const uint8_t *mask, int mode, float threshold, int B, int G,
                      uint8_t *out_mask)
{
    if (!conf32 || !mask || !out_mask || B < 0 || G < 0 || (mode != 0 && mode != 1))
        return -1;
    if (mode == 1 && !(threshold >= 0.0f && threshold <= 3.0e38f))
        return -1;
    for (int b = 0; b < B; ++b)
        for (int g = 0; g < G; ++g) {
            size_t i = (size_t)b * G + g;
            int selected = 0;
            if (mask[i] != 0) {
                double rank = 0.0;
                for (int h = 0; h < G; ++h) {
                    size_t j = (size_t)b * G + h;
                    if (mask[j] != 0 && (conf32[j] > conf32[i] || (conf32[j] == conf32[i] && h < g)))
                        rank += 1.0;
                }
                selected = mode == 0 ? (conf32[i] > threshold || rank == 0.0) : rank < floor((double)threshold);
            }
            out_mask[i] = (uint8_t)(mask[i] != 0 && !selected);
        }
    return 0;
}
